// Instantiations of the shared-producer forward kernel with skewed rows (no scan across the lanes): a measured
// alternative that only the tuning override selects, so only the plain step is instantiated.
#include "scan2d_variants.hpp"
namespace scan2d {
FwdKernel fwd_skew_kernel(bool bf16, int LG, int K, int NW, int NG, int waves, int RPB, bool sp) {
    if (sp) return nullptr;
    return bf16 ? lookup_fwd_skew_kernel<bf16_t, false>(LG, K, NW, NG, waves, RPB)
                : lookup_fwd_skew_kernel<float, false>(LG, K, NW, NG, waves, RPB);
}
}
