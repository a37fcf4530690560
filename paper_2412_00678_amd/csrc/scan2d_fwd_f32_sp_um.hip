// f32-storage instantiations of the unguarded softplus forward kernels for mask rows off the 4-byte boundaries.
#include "scan2d_variants.hpp"
namespace scan2d {
FwdKernel fwd_kernel_f32_sp_um(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi) {
    return lookup_fwd_kernel_unaligned_mask<float, false, true>(LG, K, NW, waves, exact, fast, multi);
}
}
