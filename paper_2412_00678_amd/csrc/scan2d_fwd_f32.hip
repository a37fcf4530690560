// f32-storage instantiations of the forward kernels (step given by the caller).
#include "scan2d_variants.hpp"
namespace scan2d {
FwdKernel fwd_kernel_f32_sp(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi);
FwdKernel fwd_kernel_f32_um(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi);
FwdKernel fwd_kernel_f32_sp_um(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi);
FwdKernel fwd_small_kernel_f32_sp(int KS, int NW);
FwdKernel fwd_kernel_f32(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi, bool sp, bool ma) {
    if (fast && !ma) return sp ? fwd_kernel_f32_sp_um(LG, K, NW, waves, exact, fast, multi) : fwd_kernel_f32_um(LG, K, NW, waves, exact, fast, multi);
    return sp ? fwd_kernel_f32_sp(LG, K, NW, waves, exact, fast, multi) : lookup_fwd_kernel<float, false>(LG, K, NW, waves, exact, fast, multi);
}
FwdKernel fwd_small_kernel_f32(int KS, int NW, bool sp) {
    return sp ? fwd_small_kernel_f32_sp(KS, NW) : lookup_fwd_small_kernel<float, false>(KS, NW);
}
}
