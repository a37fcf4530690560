// bf16-storage instantiations of the forward kernel.
#include "scan2d_variants.hpp"
namespace scan2d {
FwdKernel fwd_kernel_bf16(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi) {
    return lookup_fwd_kernel<bf16_t>(LG, K, NW, waves, exact, fast, multi);
}
FwdKernel fwd_small_kernel_bf16(int KS, int NW) { return lookup_fwd_small_kernel<bf16_t>(KS, NW); }
}
