"""The device gate's functions (include/freeride_device.h), compiled for the host against a stand-in for the HIP
runtime header and driven through interleavings of workgroups that a GPU may produce: late starters, workgroups
that leave before others have started, a stop between tiles.  What must hold (Section 4.5's check made on the GPU):
all workgroups of a step reach the same verdict, whatever the order; the end stamp is the time the last one left."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

SHIM = r"""
#pragma once
#include <cstdint>
#define __device__
#define __forceinline__ inline
struct Dim3 { unsigned x, y, z; };
extern thread_local Dim3 blockIdx, threadIdx;
extern unsigned long long fake_clock;
inline unsigned long long wall_clock64() { return fake_clock; }
inline unsigned atomicCAS(unsigned* p, unsigned expect, unsigned value) { unsigned old = *p; if (old == expect) *p = value; return old; }
inline unsigned long long atomicMax(unsigned long long* p, unsigned long long v) { unsigned long long old = *p; if (v > old) *p = v; return old; }
"""

DRIVER = r"""
#include <cstdio>
#include <cstdlib>
#include <vector>
#include <algorithm>
#include "freeride_device.h"
thread_local Dim3 blockIdx, threadIdx;
unsigned long long fake_clock = 0;
static unsigned rng_state = 1;
static unsigned rnd() { rng_state = rng_state * 1664525u + 1013904223u; return rng_state >> 8; }
static void as_block(unsigned b) { blockIdx = Dim3{b, 0, 0}; threadIdx = Dim3{0, 0, 0}; }
#define CHECK(c) do { if (!(c)) { printf("FAILED line %d: %s (seed %u)\n", __LINE__, #c, seed); return 1; } } while (0)

int main()
{
    for (unsigned seed = 1; seed <= 4000; ++seed) {
        rng_state = seed;
        fr_gate g{};
        fake_clock = 1000 + rnd() % 1000;
        // k_gate_open
        g.deadline_ticks = fake_clock + 5000 + rnd() % 20000; g.opened_ticks = fake_clock; g.end_ticks[0] = g.end_ticks[1] = 0; g.state = FR_GATE_OPEN; g.tiles_done = 0;
        bool closed = false;
        unsigned long long prev_end = 0;
        for (unsigned slot = 0; slot < 12; ++slot) {
            const unsigned grid = 1 + rnd() % 6, need = 200 + rnd() % 6000;
            // events: every workgroup admits, then (if admitted) leaves; any order with admit before done, the clock
            // rising all the time: workgroups may start after others have left (more workgroups than fit at once)
            std::vector<int> admitted(grid, -1), left(grid, 0);
            const bool stop_here = !closed && rnd() % 7 == 0;      // one workgroup stops the hand-out between tiles
            bool stopped = false;
            unsigned long long last_leave = 0;
            const unsigned long long expect_start = std::max(g.opened_ticks, prev_end);
            const bool expect = !closed && expect_start + need <= g.deadline_ticks;
            unsigned pending = 2 * grid;
            while (pending) {
                const unsigned b = rnd() % grid;
                fake_clock += 1 + rnd() % 400;
                as_block(b);
                if (admitted[b] < 0) {
                    admitted[b] = fr_gate_admit(&g, slot, need) ? 1 : 0;
                    CHECK(admitted[b] == (expect ? 1 : 0));               // the same verdict for every workgroup
                    if (!admitted[b]) { left[b] = 1; pending -= 2; } else pending -= 1;
                } else if (!left[b]) {
                    if (expect && stop_here && !stopped) { fr_gate_stop_short(&g, slot, 1 + rnd() % 5); stopped = true; }
                    fr_gate_done(&g, slot);
                    last_leave = fake_clock;
                    left[b] = 1; pending -= 1;
                }
            }
            if (expect) {
                CHECK(g.end_ticks[slot & 1] == last_leave);                // the stamp: when the last workgroup left
                prev_end = last_leave;
                if (stopped) { CHECK(g.state == 2 * slot + 1 && g.tiles_done >= 1); closed = true; }
            } else if (!closed) {
                CHECK(g.state == 2 * slot && g.tiles_done == 0);           // refused: recorded once, by workgroup 0
                closed = true;
            }
            if (closed) CHECK(g.state != FR_GATE_OPEN && (g.state >> 1) <= slot);   // the first such step stays on record
        }
    }
    // may_take: a tile still fits exactly up to the deadline
    {
        unsigned seed = 0;
        fr_gate g{}; g.deadline_ticks = 10000; fake_clock = 4000;
        CHECK(fr_gate_may_take(&g, 1000, 5000) && !fr_gate_may_take(&g, 1001, 5000) && fr_gate_may_take(nullptr, 1u << 30, 1u << 30));
    }
    printf("ok\n");
    return 0;
}
"""


def test_gate_verdicts_do_not_depend_on_the_order_of_workgroups(tmp_path):
    (tmp_path / "hip").mkdir()
    (tmp_path / "hip" / "hip_runtime.h").write_text(SHIM)
    (tmp_path / "driver.cpp").write_text(DRIVER)
    exe = tmp_path / "driver"
    subprocess.run(["g++", "-std=c++17", "-O1", "-I", str(tmp_path), "-I", os.path.join(ROOT, "include"),
                    str(tmp_path / "driver.cpp"), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0 and out.stdout.strip() == "ok", out.stdout + out.stderr
