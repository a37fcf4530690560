// bf16-storage instantiations of the unguarded softplus forward kernels for rows of odd width.
#include "scan2d_variants.hpp"
namespace scan2d {
FwdKernel fwd_kernel_bf16_sp_ua(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi) {
    return lookup_fwd_kernel_unaligned_mask<bf16_t, true, true>(LG, K, NW, waves, exact, fast, multi);
}
}
