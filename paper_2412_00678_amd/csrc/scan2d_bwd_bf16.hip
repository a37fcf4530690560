// bf16-storage instantiations of the backward kernels (step given by the caller).
#include "scan2d_bwd_variants.hpp"
namespace scan2d {
BwdKernels bwd_kernels_bf16_sp(int LG, int K, int NW, int waves, bool fast);
BwdKernel bwd_small_kernel_bf16_sp(int NW);
BwdKernels bwd_kernels_bf16(int LG, int K, int NW, int waves, bool fast, bool sp) {
    return sp ? bwd_kernels_bf16_sp(LG, K, NW, waves, fast) : lookup_bwd_kernels<bf16_t, false>(LG, K, NW, waves, fast);
}
BwdKernel bwd_small_kernel_bf16(int NW, bool sp) { return sp ? bwd_small_kernel_bf16_sp(NW) : lookup_bwd_small_kernel<bf16_t, false>(NW); }
}
