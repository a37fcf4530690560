// f32-storage instantiations of the small-map backward kernel that computes the step, delta = softplus(raw + bias).
#include "scan2d_bwd_variants.hpp"
namespace scan2d {
BwdKernel bwd_small_kernel_f32_sp(int NW) { return lookup_bwd_small_kernel<float, true>(NW); }
}
