// bf16-storage instantiations of the unguarded forward kernels for rows of odd width (odd 2-byte boundaries).
#include "scan2d_variants.hpp"
namespace scan2d {
FwdKernel fwd_kernel_bf16_ua(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi) {
    return lookup_fwd_kernel_unaligned_mask<bf16_t, true>(LG, K, NW, waves, exact, fast, multi);
}
}
