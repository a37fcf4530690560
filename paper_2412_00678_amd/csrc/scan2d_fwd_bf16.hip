// bf16-storage instantiations of the forward kernel.
#include "scan2d_variants.hpp"
namespace scan2d {
FwdKernel fwd_kernel_bf16(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi) {
    return lookup_fwd_kernel<bf16_t>(LG, K, NW, waves, exact, fast, multi);
}
}
