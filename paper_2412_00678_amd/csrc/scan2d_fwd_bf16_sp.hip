// bf16-storage instantiations of the forward kernels that compute the step, delta = softplus(raw + bias).
#include "scan2d_variants.hpp"
namespace scan2d {
FwdKernel fwd_kernel_bf16_sp(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi) {
    return lookup_fwd_kernel<bf16_t, true>(LG, K, NW, waves, exact, fast, multi);
}
FwdKernel fwd_small_kernel_bf16_sp(int KS, int NW) { return lookup_fwd_small_kernel<bf16_t, true>(KS, NW); }
}
