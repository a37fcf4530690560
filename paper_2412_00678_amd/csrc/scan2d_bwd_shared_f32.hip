// f32-storage instantiations of the backward main sweeps that share the per-position work through LDS.
#include "scan2d_bwd_variants.hpp"
namespace scan2d {
BwdKernels bwd_shared_kernels_f32(int LG, int K, int NW, int NG, int waves, int W, bool sp) {
    return sp ? lookup_bwd_shared_kernels<float, true>(LG, K, NW, NG, waves, W)
              : lookup_bwd_shared_kernels<float, false>(LG, K, NW, NG, waves, W);
}
}
