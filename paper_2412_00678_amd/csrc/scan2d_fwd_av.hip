// Forward instantiations with an independent decay for the column recurrence (the supplement's A-bar ablation).
#include "scan2d_variants.hpp"
namespace scan2d {
FwdKernel fwd_kernel_av_f32() { return scan2d_fwd_kernel<float, 16, 4, 4, 4, false, false, true, false, true, false, true>; }
FwdKernel fwd_kernel_av_bf16() { return scan2d_fwd_kernel<bf16_t, 16, 4, 4, 4, false, false, true, false, true, false, true>; }
}
