// bf16-storage instantiations of the forward kernels that share the per-position work through LDS.
#include "scan2d_variants.hpp"
namespace scan2d {
FwdKernel fwd_shared_kernel_bf16(int LG, int K, int NW, int NG, int waves, int RPB, bool sp, bool ua) {
    if (ua) return sp ? lookup_fwd_shared_kernel<bf16_t, true, true>(LG, K, NW, NG, waves, RPB)
                      : lookup_fwd_shared_kernel<bf16_t, false, true>(LG, K, NW, NG, waves, RPB);
    return sp ? lookup_fwd_shared_kernel<bf16_t, true, false>(LG, K, NW, NG, waves, RPB)
              : lookup_fwd_shared_kernel<bf16_t, false, false>(LG, K, NW, NG, waves, RPB);
}
}
