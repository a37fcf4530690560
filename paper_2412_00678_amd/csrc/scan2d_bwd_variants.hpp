// The backward kernel variants that are compiled: (LG, K, NW, WAVES, RB, PF), RB = rows per
// band, PF = next-row prefetch.  RB * NW * K bounds the rebuilt states and the channel-sum
// accumulators held in VGPRs.
#pragma once

#include "scan2d_bwd_kernels.hpp"
#include "scan2d_bwd_small.hpp"

namespace scan2d {

#define SCAN2D_BWD_VARIANTS(X)                                             \
    X(16, 4, 1, 4, 4, true) X(16, 8, 1, 4, 4, true) X(16, 12, 1, 4, 4, false) X(16, 16, 1, 4, 2, true) \
    X(16, 4, 4, 4, 2, true) X(16, 8, 4, 4, 1, true)                                                   \
    X(64, 4, 2, 8, 4, false) X(64, 8, 2, 8, 2, false) X(64, 16, 4, 4, 1, false)                           \
    X(64, 4, 4, 16, 2, false) X(64, 8, 4, 16, 1, false) X(64, 4, 1, 16, 2, false)

using BwdKernel = void (*)(const BwdArgs);
struct BwdKernels { BwdKernel ckpt = nullptr; BwdKernel main = nullptr; int RB = 0; int ckpt_NW = 0; };

// sp: the instantiations that compute the step themselves (softplus of the raw projection).
BwdKernels bwd_kernels_f32(int LG, int K, int NW, int waves, bool fast, bool sp);
BwdKernels bwd_kernels_bf16(int LG, int K, int NW, int waves, bool fast, bool sp);

template <typename T, bool SP>
inline BwdKernels lookup_bwd_kernels(int LG, int K, int NW, int waves, bool fast) {
    BwdKernels r;
#define SCAN2D_X(lg, k, nw, wv, rb, pf)                                                                 \
    if (LG == lg && K == k && NW == nw && waves == wv) {                                                \
        constexpr int cnw = (lg == 16 && nw == 1) ? 2 : nw;   /* the checkpoint sweep has registers to spare */ \
        r.ckpt = fast ? scan2d_bwd_ckpt_kernel<T, lg, k, cnw, wv, rb, true, SP> : scan2d_bwd_ckpt_kernel<T, lg, k, cnw, wv, rb, false, SP>; \
        r.ckpt_NW = cnw;                                                                                \
        r.main = fast ? scan2d_bwd_main_kernel<T, lg, k, nw, wv, rb, true, pf, SP> : scan2d_bwd_main_kernel<T, lg, k, nw, wv, rb, false, pf, SP>; \
        r.RB = rb;                                                                                      \
    }
    SCAN2D_BWD_VARIANTS(SCAN2D_X)
#undef SCAN2D_X
    return r;
}

// Small maps (W, H, N <= 16): one wavefront per map, NW = states per lane group of its four.
BwdKernel bwd_small_kernel_f32(int NW, bool sp);
BwdKernel bwd_small_kernel_bf16(int NW, bool sp);

template <typename T, bool SP>
inline BwdKernel lookup_bwd_small_kernel(int NW) {
    if (NW == 1) return scan2d_bwd_small_kernel<T, 1, SP>;
    if (NW == 2) return scan2d_bwd_small_kernel<T, 2, SP>;
    if (NW == 4) return scan2d_bwd_small_kernel<T, 4, SP>;
    return nullptr;
}

}  // namespace scan2d
