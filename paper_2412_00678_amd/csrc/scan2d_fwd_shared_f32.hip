// f32-storage instantiations of the forward kernels that share the per-position work through LDS.
#include "scan2d_variants.hpp"
namespace scan2d {
FwdKernel fwd_shared_kernel_f32(int LG, int K, int NW, int NG, int waves, int RPB, bool sp) {
    return sp ? lookup_fwd_shared_kernel<float, true, false>(LG, K, NW, NG, waves, RPB)
              : lookup_fwd_shared_kernel<float, false, false>(LG, K, NW, NG, waves, RPB);
}
}
