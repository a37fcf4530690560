// f32-storage instantiations of the columns-first forward kernels (shared-producer form).
#include "scan2d_variants.hpp"
namespace scan2d {
FwdKernel fwd_shared_kernel_f32_cf(int LG, int K, int NW, int NG, int waves, int RPB, bool sp) {
    return sp ? lookup_fwd_shared_kernel<float, true, false, true>(LG, K, NW, NG, waves, RPB)
              : lookup_fwd_shared_kernel<float, false, false, true>(LG, K, NW, NG, waves, RPB);
}
}
