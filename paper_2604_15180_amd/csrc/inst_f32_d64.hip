// Kernel instantiations for f32 inputs, head dim 64.
// fp32 inputs: every product on the fp32 MFMA (32x32x2), no copies.
#include "ops.hpp"

namespace ea {
int run_f32_d64(bool is_bwd, const Params& p, bool rebuild_mask, void* const copies[4], hipStream_t s) {
    return dispatch_alpha<F32, F32, 64>(is_bwd, p, rebuild_mask, copies, s);
}
}  // namespace ea
