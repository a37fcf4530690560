// bf16-storage instantiations of the columns-first forward kernels (shared-producer form).
#include "scan2d_variants.hpp"
namespace scan2d {
FwdKernel fwd_shared_kernel_bf16_cf(int LG, int K, int NW, int NG, int waves, int RPB, bool sp, bool ua) {
    if (ua) return sp ? lookup_fwd_shared_kernel<bf16_t, true, true, true>(LG, K, NW, NG, waves, RPB)
                      : lookup_fwd_shared_kernel<bf16_t, false, true, true>(LG, K, NW, NG, waves, RPB);
    return sp ? lookup_fwd_shared_kernel<bf16_t, true, false, true>(LG, K, NW, NG, waves, RPB)
              : lookup_fwd_shared_kernel<bf16_t, false, false, true>(LG, K, NW, NG, waves, RPB);
}
}
