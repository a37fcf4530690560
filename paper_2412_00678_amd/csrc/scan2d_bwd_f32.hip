// f32-storage instantiations of the backward kernels.
#include "scan2d_bwd_variants.hpp"
namespace scan2d {
BwdKernels bwd_kernels_f32(int LG, int K, int NW, int waves, bool fast) { return lookup_bwd_kernels<float>(LG, K, NW, waves, fast); }
BwdKernel bwd_small_kernel_f32(int NW) { return lookup_bwd_small_kernel<float>(NW); }
}
