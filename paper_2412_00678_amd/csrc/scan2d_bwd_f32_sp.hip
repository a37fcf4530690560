// f32-storage instantiations of the backward kernels for the softplus step, delta = softplus(raw + bias).
#include "scan2d_bwd_variants.hpp"
namespace scan2d {
BwdKernels bwd_kernels_f32_sp(int LG, int K, int NW, int waves, bool fast) { return lookup_bwd_kernels<float, true>(LG, K, NW, waves, fast); }
BwdKernel bwd_small_kernel_f32_sp(int NW) { return lookup_bwd_small_kernel<float, true>(NW); }
}
