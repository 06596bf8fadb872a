/*
 * freeride_device.h -- device-side half of the program-directed time limit (FreeRide, arXiv 2409.06941,
 * Section 4.5: a side task runs its next step only if the time left in the bubble is enough for it).
 *
 * The host plans steps against a cost model and enqueues them ahead of the GPU.  With fr_config.device_gate set
 * the same check is made again on the GPU's own timeline, by the kernels themselves:
 *   - when a step's kernel starts: can the step (or, for a kernel that hands its tiles out in rounds, its first
 *     round) still end before the bubble does?  If not the step is REFUSED: the kernel returns before touching
 *     any task state;
 *   - between the tiles of a kernel that hands out its tiles (fr_gate_may_take): is there still time for one more
 *     tile?  If not the kernel stops handing out, the workgroups finish the tiles they hold and leave, and the
 *     step has STOPPED SHORT after a whole number of its tiles, which the gate records;
 *   - every step enqueued behind a refused or short step does nothing.
 * The runtime reads the record once the stream has drained and rewinds the task to the first tile that was not
 * done (fr_task_ops.rewind), so the work is taken up again in a later bubble.
 *
 * All workgroups of a kernel must reach the same verdict at its start, so that verdict is a pure function of memory
 * no workgroup of the same kernel writes: the step is taken to start when the previous step ended or when the gate
 * was opened, whichever is later, and the end stamps of consecutive steps live in two words used in turn - step
 * s reads the word of step s - 1 and its own workgroups write the other one (each leaving workgroup raises it to its
 * clock, so the stamp is the time the last of them left).  The one word a kernel may both read and write is `state`,
 * and a workgroup that finds there that its own step stopped short carries on: the closure is its own kernel's doing
 * and concerns the tiles not yet handed out, not the tile of the first round it is about to start.
 * Steps of one context run one after the other on the side stream, which is what makes this sound.
 *
 * For HIP device code only.  A task's step kernel calls fr_gate_admit first thing, all threads of every
 * workgroup, returns when it says false, and calls fr_gate_done last thing.  The arguments come from the fr_step
 * handed to run_step.  A step made of several kernels admits in the first and is done in the last.
 */
#ifndef FREERIDE_DEVICE_H
#define FREERIDE_DEVICE_H

#include <hip/hip_runtime.h>

#define FR_GATE_OPEN 0xffffffffu

struct fr_gate {
    unsigned long long deadline_ticks;   /* wall_clock64() value by which a step must have ended               */
    unsigned long long opened_ticks;     /* clock when the gate was opened for the current bubble              */
    unsigned long long end_ticks[2];     /* [s & 1]: clock when the last workgroup of step s left              */
    unsigned int state;                  /* FR_GATE_OPEN, or 2 * slot (+ 1 if it stopped short, + 0 if it was refused)
                                            of the first step that did not run in full since the gate was opened:
                                            later steps do nothing                                              */
    unsigned int tiles_done;             /* of a step that stopped short: its first tiles_done tiles were completed */
};

/* gate == NULL admits.  need_ticks: what must still fit, in ticks of wall_clock64(): the whole step, or the first
   round of a kernel that hands its tiles out. */
__device__ __forceinline__ bool fr_gate_admit(fr_gate* gate, unsigned int slot, unsigned int need_ticks)
{
    if (!gate) return true;
    const unsigned int state = gate->state;
    if (state != FR_GATE_OPEN) return state == 2u * slot + 1u;     /* closed by an earlier step, or by this one: see above */
    const unsigned long long prev_end = gate->end_ticks[(slot + 1u) & 1u];
    const unsigned long long start = gate->opened_ticks > prev_end ? gate->opened_ticks : prev_end;
    const bool admit = start + need_ticks <= gate->deadline_ticks;
    if (!admit && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x == 0 && threadIdx.y == 0 && threadIdx.z == 0) {
        /* the one writer; the other workgroups of this kernel reach the same verdict from the clock values, which
           nobody changes while a refused kernel runs, or already read the refusal in `state` */
        gate->tiles_done = 0u;
        gate->state = 2u * slot;
    }
    return admit;
}

/* Between tiles, one thread of a workgroup that is about to take another tile: true if a tile of tile_ticks can
   still end `ahead_ticks + tile_ticks` from now before the deadline (ahead_ticks: what the workgroup still has to
   do before it would start that tile).  gate == NULL: true. */
__device__ __forceinline__ bool fr_gate_may_take(const fr_gate* gate, unsigned int ahead_ticks, unsigned int tile_ticks)
{
    return !gate || wall_clock64() + ahead_ticks + tile_ticks <= gate->deadline_ticks;
}

/* The step `slot` stops after its first `tiles_done` tiles (one thread of one workgroup, once per kernel).  Only the
   first such step since the gate was opened is recorded: that is where the task is taken up again. */
__device__ __forceinline__ void fr_gate_stop_short(fr_gate* gate, unsigned int slot, unsigned int tiles_done)
{
    if (!gate) return;
    if (atomicCAS(&gate->state, FR_GATE_OPEN, 2u * slot + 1u) == FR_GATE_OPEN) gate->tiles_done = tiles_done;
}

/* Last thing in a step's (last) kernel, all workgroups.  An admitted step leaves its end stamp for the next one. */
__device__ __forceinline__ void fr_gate_done(fr_gate* gate, unsigned int slot)
{
    if (gate && threadIdx.x == 0 && threadIdx.y == 0 && threadIdx.z == 0) atomicMax(&gate->end_ticks[slot & 1u], wall_clock64());
}

#endif /* FREERIDE_DEVICE_H */
