// What the host side (api.hip) and the per-type kernel translation units share: the entry
// that runs one forward or backward kernel sequence for a given (input type, head dim), and the
// hooks those sequences call back into (HIP error slot, per-kernel timing).
// The kernels are instantiated in one translation unit per (type, head dim): they compile in
// parallel, and each type gets the code-generation flags that suit it.
#pragma once
#include "../../include/entmax_attn_aids.h"
#include "common.hpp"

namespace ea {

constexpr int NBINS = 63;    // histogram bins B per unit (Sec. 3.1): bracket width 1/63 after the histogram solve
constexpr int MAX_SWEEPS = 12;

void set_last_hip_error(int e);
// Records a HIP event on `s` before (which = 0) or after (which = 1) the kernels of timer slot
// `slot`; does nothing unless timing was switched on for the call in flight.
void timer_mark(int slot, int which, hipStream_t s);
// Opens the timer row of a new library call (no-op unless timing is switched on).
void timer_begin();

struct ScopedKernelTime {
    int slot; hipStream_t s;
    ScopedKernelTime(int slot_, hipStream_t s_) : slot(slot_), s(s_) { timer_mark(slot, 0, s); }
    ~ScopedKernelTime() { timer_mark(slot, 1, s); }
};

// `copies`: workspace room for K, Q, V, dO in the stage-2 element type (backward, bf16 inputs)
#define EA_DECLARE_RUN(name) \
    int name(bool is_bwd, const Params& p, bool rebuild_mask, void* const copies[4], hipStream_t s)
EA_DECLARE_RUN(run_bf16_d64);
EA_DECLARE_RUN(run_bf16_d128);
EA_DECLARE_RUN(run_f32_d64);
EA_DECLARE_RUN(run_f32_d128);

}  // namespace ea
