// f32-storage instantiations of the backward kernels (step given by the caller).
#include "scan2d_bwd_variants.hpp"
namespace scan2d {
BwdKernel bwd_small_kernel_f32_sp(int NW);
// sp: with f32 storage the banded sweeps never compute the step themselves (a kernel of its own writes it
// first, see scan2d_bwd.hip); only the small-map kernel has such instantiations.
BwdKernels bwd_kernels_f32(int LG, int K, int NW, int waves, bool fast, bool sp) {
    return sp ? BwdKernels{} : lookup_bwd_kernels<float, false>(LG, K, NW, waves, fast);
}
BwdKernel bwd_small_kernel_f32(int NW, bool sp) { return sp ? bwd_small_kernel_f32_sp(NW) : lookup_bwd_small_kernel<float, false>(NW); }
}
