// f32-storage instantiations of the backward kernels (step given by the caller).
#include "scan2d_bwd_variants.hpp"
namespace scan2d {
BwdKernels bwd_kernels_f32_sp(int LG, int K, int NW, int waves, bool fast);
BwdKernel bwd_small_kernel_f32_sp(int NW);
BwdKernels bwd_kernels_f32(int LG, int K, int NW, int waves, bool fast, bool sp) {
    return sp ? bwd_kernels_f32_sp(LG, K, NW, waves, fast) : lookup_bwd_kernels<float, false>(LG, K, NW, waves, fast);
}
BwdKernel bwd_small_kernel_f32(int NW, bool sp) { return sp ? bwd_small_kernel_f32_sp(NW) : lookup_bwd_small_kernel<float, false>(NW); }
}
