// Kernel instantiations for bf16 inputs, head dim 128.
// bf16 inputs: the forward scores (Q K^T) run on bf16 MFMA straight from the inputs.  Every
// second-stage product (P V, dS K, P^T dO, dS^T Q) and the whole backward run on fp16 MFMA
// from fp16 copies: P lies in [0,1] and dO is divided by max|dO| first, so fp16's range
// suffices and its 3 extra mantissa bits keep the rounding of P and dS well inside the
// tolerances; bf16 values convert to fp16 exactly while 2^-17 <= |x| < 65504 (smaller ones
// within 2^-25 absolute; larger ones are outside this library's domain).
#include "ops.hpp"

namespace ea {
int run_bf16_d128(bool is_bwd, const Params& p, bool rebuild_mask, void* const copies[4], hipStream_t s) {
    return dispatch_alpha<Bf16, F16, 128>(is_bwd, p, rebuild_mask, copies, s);
}
}  // namespace ea
