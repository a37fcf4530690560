// bf16-storage instantiations of the backward kernels that compute the step, delta = softplus(raw + bias).
#include "scan2d_bwd_variants.hpp"
namespace scan2d {
BwdKernels bwd_kernels_bf16_sp(int LG, int K, int NW, int waves, bool fast) { return lookup_bwd_kernels<bf16_t, true>(LG, K, NW, waves, fast); }
BwdKernel bwd_small_kernel_bf16_sp(int NW) { return lookup_bwd_small_kernel<bf16_t, true>(NW); }
}
