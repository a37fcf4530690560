// f32-storage instantiations of the forward kernel.
#include "scan2d_variants.hpp"
namespace scan2d {
FwdKernel fwd_kernel_f32(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi) {
    return lookup_fwd_kernel<float>(LG, K, NW, waves, exact, fast, multi);
}
FwdKernel fwd_small_kernel_f32(int KS, int NW) { return lookup_fwd_small_kernel<float>(KS, NW); }
}
