// The (LG, K, NW, WAVES) kernel variants that are compiled, and the lookup used by the dispatcher.
//   LG    : lanes per lane group (16 = one DPP row, 32 = half a wavefront, 64 = a wavefront)
//   K     : consecutive columns per lane
//   NW    : states per lane
//   WAVES : wavefronts per workgroup
// K * NW <= 64 bounds the persistent column state held in VGPRs; the 8- and 16-wave forms are
// limited to the variants whose register count allows that many waves per SIMD.
#pragma once

#include "scan2d_fwd.hpp"
#include "scan2d_fwd_shared.hpp"
#include "scan2d_fwd_small.hpp"

namespace scan2d {

#define SCAN2D_FWD_VARIANTS(X)                                                  \
    X(16, 4, 1, 4) X(16, 4, 2, 4) X(16, 4, 4, 4) X(16, 4, 8, 4) X(16, 4, 16, 4) \
    X(16, 8, 1, 4) X(16, 8, 2, 4) X(16, 8, 4, 4) X(16, 8, 8, 4)                 \
    X(16, 12, 1, 4) X(16, 12, 2, 4) X(16, 12, 4, 4)                             \
    X(16, 16, 1, 4) X(16, 16, 2, 4) X(16, 16, 4, 4)                             \
    X(64, 4, 1, 4) X(64, 4, 2, 4) X(64, 4, 4, 4) X(64, 4, 8, 4) X(64, 4, 16, 4) \
    X(64, 8, 1, 4) X(64, 8, 2, 4) X(64, 8, 4, 4) X(64, 8, 8, 4)                 \
    X(64, 16, 1, 4) X(64, 16, 2, 4) X(64, 16, 4, 4)                             \
    X(64, 4, 1, 8) X(64, 4, 2, 8) X(64, 8, 1, 8) X(64, 8, 2, 8) X(64, 16, 1, 8) \
    X(64, 4, 1, 16) X(64, 8, 1, 16)                                             \
    X(32, 4, 1, 8) X(32, 4, 2, 4) X(32, 4, 4, 4) X(32, 8, 1, 8) X(32, 8, 2, 4) X(32, 8, 2, 8) X(32, 8, 4, 4)

// Variants that also exist for N not divisible by NW (the last lane group idles some states).
#define SCAN2D_FWD_RAGGED_VARIANTS(X) X(16, 4, 4, 4) X(16, 8, 4, 4) X(16, 12, 4, 4) X(16, 16, 4, 4)

// Variants that also exist for maps wider than one panel (guarded accesses, any W); single-panel maps
// always take the unguarded variants.
#define SCAN2D_FWD_MULTI_VARIANTS(X)                                            \
    X(64, 4, 1, 4) X(64, 4, 2, 4) X(64, 4, 4, 4) X(64, 4, 8, 4) X(64, 4, 16, 4) \
    X(64, 4, 1, 8) X(64, 4, 2, 8) X(64, 4, 1, 16) X(16, 4, 4, 4)

using FwdKernel = void (*)(const FwdArgs);

// Variants of the form that shares the per-position work of a map through LDS: (LG, K, NW, NG, WAVES, RPB);
// NG = N / NW lane groups per map, RPB rows between two barriers.
#define SCAN2D_FWD_SHARED_VARIANTS(X)                                                     \
    X(64, 4, 2, 8, 8, 4) X(64, 4, 2, 8, 8, 8) X(64, 4, 1, 16, 16, 4)                      \
    /* 257 to 1024 columns */ X(64, 8, 1, 16, 16, 2) X(64, 8, 2, 8, 8, 2) X(64, 12, 2, 8, 8, 2) X(64, 16, 2, 8, 8, 2) \
    X(16, 12, 1, 16, 4, 4) X(16, 12, 2, 8, 4, 2) X(16, 8, 1, 16, 4, 4) X(16, 8, 2, 8, 4, 2) \
    X(16, 4, 1, 16, 4, 4) X(16, 4, 2, 8, 4, 4) X(16, 4, 4, 4, 4, 4) X(16, 4, 8, 2, 4, 4)   \
    /* N = 8 */ X(64, 4, 1, 8, 8, 4) X(16, 4, 1, 8, 4, 4) X(16, 4, 2, 4, 4, 4) X(16, 8, 1, 8, 4, 4) X(16, 12, 1, 8, 4, 4) \
    /* N = 4 */ X(64, 4, 1, 4, 4, 4) X(16, 4, 1, 4, 4, 4) X(16, 8, 1, 4, 4, 4)             \
    /* N = 32 */ X(64, 4, 2, 16, 16, 4) X(64, 4, 4, 8, 8, 4) X(16, 4, 2, 16, 4, 4) X(16, 8, 2, 16, 4, 4) X(16, 4, 4, 8, 4, 4) \
    /* N = 64 */ X(64, 4, 4, 16, 16, 4) X(16, 4, 4, 16, 4, 4) X(16, 8, 4, 16, 4, 2)

// Tilings of the same kernel with skewed rows (lane l of a group on row t - l: no scan across the lanes), all with
// one state per lane: (LG, K, NW, NG, WAVES, RPB).  Only the tuning override selects them.
#define SCAN2D_FWD_SKEW_VARIANTS(X) \
    X(16, 16, 1, 16, 4, 4) X(16, 8, 1, 16, 4, 4) X(64, 4, 1, 16, 16, 4)
// nullptr when the tiling is not compiled
FwdKernel fwd_skew_kernel(bool bf16, int LG, int K, int NW, int NG, int waves, int RPB, bool sp);

FwdKernel fwd_shared_kernel_f32(int LG, int K, int NW, int NG, int waves, int RPB, bool sp);
FwdKernel fwd_shared_kernel_bf16(int LG, int K, int NW, int NG, int waves, int RPB, bool sp, bool ua);
// The columns-first instantiations of the same tilings.
FwdKernel fwd_shared_kernel_f32_cf(int LG, int K, int NW, int NG, int waves, int RPB, bool sp);
FwdKernel fwd_shared_kernel_bf16_cf(int LG, int K, int NW, int NG, int waves, int RPB, bool sp, bool ua);

// The instantiations that also apply the block's output gate (softplus step, rows first).
FwdKernel fwd_shared_kernel_gate_f32(int LG, int K, int NW, int NG, int waves, int RPB);
FwdKernel fwd_shared_kernel_gate_bf16(int LG, int K, int NW, int NG, int waves, int RPB, bool ua);

template <typename T, bool SP, bool UA, bool CF = false, bool GATE = false>
inline FwdKernel lookup_fwd_shared_kernel(int LG, int K, int NW, int NG, int waves, int RPB) {
#define SCAN2D_X(lg, k, nw, ng, wv, rpb) \
    if (LG == lg && K == k && NW == nw && NG == ng && waves == wv && RPB == rpb) return scan2d_fwd_shared_kernel<T, lg, k, nw, ng, wv, rpb, SP, UA, 0, CF, false, GATE>;
    SCAN2D_FWD_SHARED_VARIANTS(SCAN2D_X)
#undef SCAN2D_X
    return nullptr;
}

template <typename T, bool SP>
inline FwdKernel lookup_fwd_skew_kernel(int LG, int K, int NW, int NG, int waves, int RPB) {
#define SCAN2D_X(lg, k, nw, ng, wv, rpb) \
    if (LG == lg && K == k && NW == nw && NG == ng && waves == wv && RPB == rpb) return scan2d_fwd_shared_kernel<T, lg, k, nw, ng, wv, rpb, SP, false, 0, false, false, false, true>;
    SCAN2D_FWD_SKEW_VARIANTS(SCAN2D_X)
#undef SCAN2D_X
    return nullptr;
}

// Returns nullptr when the variant is not compiled.
// sp: the instantiations that compute the step themselves (softplus of the raw projection).
// ma: mask rows start on 4-byte boundaries (no mask, or W a multiple of 4); the instantiations for the
//     other case exist for the unguarded variants.
// ua (bf16 only): tensor rows start on odd 2-byte boundaries (odd W); exists for the unguarded variants.
FwdKernel fwd_kernel_f32(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi, bool sp, bool ma);
FwdKernel fwd_kernel_bf16(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi, bool sp, bool ma, bool ua = false);

// Unguarded variants for mask rows that do not start on 4-byte boundaries, and (UA, bf16 only) for
// tensor rows that do not either.
template <typename T, bool UA = false, bool SP = false>
inline FwdKernel lookup_fwd_kernel_unaligned_mask(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi);

// Independent vertical decay (AV): one guarded, multi-panel capable, ragged-N capable instantiation per storage
// type covers every shape (an ablation mode, not a tuned path).
FwdKernel fwd_kernel_av_f32();
FwdKernel fwd_kernel_av_bf16();

// Narrow maps (W <= 32): KS columns per lane, NW = states per lane group of the wave's four.
FwdKernel fwd_small_kernel_f32(int KS, int NW, bool sp);
// maps of at most 16 x 16 positions and 16 states, one workgroup per map, both recurrences as parallel scans
// (scan2d_fwd_tile16.hip)
FwdKernel fwd_tile16_kernel(int dtype, bool sp);
FwdKernel fwd_small_kernel_bf16(int KS, int NW, bool sp);

template <typename T, bool SP>
inline FwdKernel lookup_fwd_small_kernel(int KS, int NW) {
#define SCAN2D_X(ks, nw, pd) \
    if (KS == ks && NW == nw) return scan2d_fwd_small_kernel<T, ks, nw, pd, SP>;
    SCAN2D_X(1, 1, 4) SCAN2D_X(1, 2, 4) SCAN2D_X(1, 4, 4) SCAN2D_X(1, 8, 2) SCAN2D_X(1, 16, 2)
    SCAN2D_X(2, 1, 4) SCAN2D_X(2, 2, 4) SCAN2D_X(2, 4, 4) SCAN2D_X(2, 8, 2) SCAN2D_X(2, 16, 1)
#undef SCAN2D_X
    return nullptr;
}

template <typename T, bool SP>
inline FwdKernel lookup_fwd_kernel(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi) {
#define SCAN2D_X(lg, k, nw, wv) \
    if (exact && fast && !multi && LG == lg && K == k && NW == nw && waves == wv) return scan2d_fwd_kernel<T, lg, k, nw, wv, true, true, false, SP>;
    SCAN2D_FWD_VARIANTS(SCAN2D_X)
#undef SCAN2D_X
#define SCAN2D_X(lg, k, nw, wv) \
    if (!exact && fast && !multi && LG == lg && K == k && NW == nw && waves == wv) return scan2d_fwd_kernel<T, lg, k, nw, wv, false, true, false, SP>;
    SCAN2D_FWD_RAGGED_VARIANTS(SCAN2D_X)
#undef SCAN2D_X
#define SCAN2D_X(lg, k, nw, wv) \
    if (exact && !fast && multi && LG == lg && K == k && NW == nw && waves == wv) return scan2d_fwd_kernel<T, lg, k, nw, wv, true, false, true, SP>;
    SCAN2D_FWD_MULTI_VARIANTS(SCAN2D_X)
#undef SCAN2D_X
    if (!exact && !fast && multi && LG == 16 && K == 4 && NW == 4 && waves == 4)
        return scan2d_fwd_kernel<T, 16, 4, 4, 4, false, false, true, SP>;
    return nullptr;
}

template <typename T, bool UA, bool SP>
inline FwdKernel lookup_fwd_kernel_unaligned_mask(int LG, int K, int NW, int waves, bool exact, bool fast, bool multi) {
#define SCAN2D_X(lg, k, nw, wv) \
    if (exact && fast && !multi && LG == lg && K == k && NW == nw && waves == wv) return scan2d_fwd_kernel<T, lg, k, nw, wv, true, true, false, SP, false, UA>;
    SCAN2D_FWD_VARIANTS(SCAN2D_X)
#undef SCAN2D_X
#define SCAN2D_X(lg, k, nw, wv) \
    if (!exact && fast && !multi && LG == lg && K == k && NW == nw && waves == wv) return scan2d_fwd_kernel<T, lg, k, nw, wv, false, true, false, SP, false, UA>;
    SCAN2D_FWD_RAGGED_VARIANTS(SCAN2D_X)
#undef SCAN2D_X
    return nullptr;
}

}  // namespace scan2d
