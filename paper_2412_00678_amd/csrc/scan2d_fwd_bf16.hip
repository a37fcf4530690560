// bf16-storage instantiations of the forward kernels (step given by the caller).
#include "scan2d_variants.hpp"
namespace scan2d {
FwdKernel fwd_kernel_bf16_sp(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi);
FwdKernel fwd_kernel_bf16_um(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi);
FwdKernel fwd_kernel_bf16_ua(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi);
FwdKernel fwd_kernel_bf16_sp_um(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi);
FwdKernel fwd_kernel_bf16_sp_ua(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi);
FwdKernel fwd_small_kernel_bf16_sp(int KS, int NW);
FwdKernel fwd_kernel_bf16(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi, bool sp, bool ma, bool ua) {
    if (fast && ua) return sp ? fwd_kernel_bf16_sp_ua(LG, K, NW, waves, exact, fast, multi) : fwd_kernel_bf16_ua(LG, K, NW, waves, exact, fast, multi);
    if (fast && !ma) return sp ? fwd_kernel_bf16_sp_um(LG, K, NW, waves, exact, fast, multi) : fwd_kernel_bf16_um(LG, K, NW, waves, exact, fast, multi);
    return sp ? fwd_kernel_bf16_sp(LG, K, NW, waves, exact, fast, multi) : lookup_fwd_kernel<bf16_t, false>(LG, K, NW, waves, exact, fast, multi);
}
FwdKernel fwd_small_kernel_bf16(int KS, int NW, bool sp) {
    return sp ? fwd_small_kernel_bf16_sp(KS, NW) : lookup_fwd_small_kernel<bf16_t, false>(KS, NW);
}
}
