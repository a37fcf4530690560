// f32-storage instantiations of the columns-first backward sweeps (16-lane tilings, shared-producer main sweep).
#include "scan2d_bwd_variants.hpp"
namespace scan2d {
BwdKernels bwd_shared_kernels_f32_cf(int LG, int K, int NW, int NG, int waves, int W, bool sp) {
    return sp ? lookup_bwd_shared_kernels<float, true, true>(LG, K, NW, NG, waves, W)
              : lookup_bwd_shared_kernels<float, false, true>(LG, K, NW, NG, waves, W);
}
}
