/*
 * freeride_device.h -- device-side half of the program-directed time limit (FreeRide, arXiv 2409.06941,
 * Section 4.5: a side task runs its next step only if the time left in the bubble is enough for it).
 *
 * The host plans steps against a cost model and enqueues them ahead of the GPU.  With fr_config.device_gate set
 * every step is also checked on the GPU's own timeline when its kernel starts: can it still end before the
 * bubble does?  A step that cannot is refused: its kernel returns before touching any task state, and so does
 * every step enqueued behind it.  The runtime learns which step was refused first and rewinds the task there
 * (fr_task_ops.rewind), so the work is done again in a later bubble.
 *
 * All workgroups of a step must reach the same verdict, so the verdict is a pure function of memory that is
 * fixed before the step's kernel starts: the step is taken to start when the previous step ended (its last
 * workgroup stored the clock on its way out) or when the gate was opened, whichever is later.  No atomics, no
 * waiting.  Steps of one context run one after the other on the side stream, which is what makes this sound.
 *
 * For HIP device code only.  A task's step kernel calls fr_gate_admit first thing, all threads of every
 * workgroup, returns when it says false, and calls fr_gate_done last thing.  The arguments come from the fr_step
 * handed to run_step.  A step made of several kernels admits in the first and is done in the last.
 */
#ifndef FREERIDE_DEVICE_H
#define FREERIDE_DEVICE_H

#include <hip/hip_runtime.h>

struct fr_gate {
    unsigned long long deadline_ticks;   /* wall_clock64() value by which a step must have ended               */
    unsigned long long opened_ticks;     /* clock when the gate was opened for the current bubble              */
    unsigned long long last_end_ticks;   /* clock when the latest admitted step ended                          */
    unsigned int closed;                 /* nonzero once a step was refused: every later step is refused too   */
    unsigned int first_refused;          /* slot of the first step refused since the gate was opened;
                                            0xffffffff: none                                                   */
};

/* gate == NULL admits. */
__device__ __forceinline__ bool fr_gate_admit(fr_gate* gate, unsigned int slot, unsigned int need_ticks)
{
    if (!gate) return true;
    const unsigned long long start = gate->opened_ticks > gate->last_end_ticks ? gate->opened_ticks : gate->last_end_ticks;
    const bool admit = gate->closed == 0u && start + need_ticks <= gate->deadline_ticks;
    if (!admit && gate->closed == 0u && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 &&
        threadIdx.x == 0 && threadIdx.y == 0 && threadIdx.z == 0) {
        /* the one writer; the other workgroups of this kernel may still read closed == 0 and reach the same
           verdict from the clock values, which nobody changes while a refused kernel runs */
        /* (no fence between the two stores: their readers - later kernels on the stream, and the host once the
           stream has drained - only look after this kernel has ended) */
        gate->first_refused = slot;
        gate->closed = 1u;
    }
    return admit;
}

__device__ __forceinline__ void fr_gate_done(fr_gate* gate)
{
    if (gate && blockIdx.x == gridDim.x - 1 && blockIdx.y == gridDim.y - 1 && blockIdx.z == gridDim.z - 1 &&
        threadIdx.x == 0 && threadIdx.y == 0 && threadIdx.z == 0)
        gate->last_end_ticks = wall_clock64();
}

#endif /* FREERIDE_DEVICE_H */
