// f32-storage instantiations of the forward kernels that compute the step, delta = softplus(raw + bias).
#include "scan2d_variants.hpp"
namespace scan2d {
FwdKernel fwd_kernel_f32_sp(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi) {
    return lookup_fwd_kernel<float, true>(LG, K, NW, waves, exact, fast, multi);
}
FwdKernel fwd_small_kernel_f32_sp(int KS, int NW) { return lookup_fwd_small_kernel<float, true>(KS, NW); }
}
