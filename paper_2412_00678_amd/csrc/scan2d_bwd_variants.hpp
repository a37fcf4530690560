// The backward kernel variants that are compiled: (LG, K, NW, WAVES, RB, PF), RB = rows per
// band, PF = next-row prefetch.  RB * NW * K bounds the rebuilt states and the channel-sum
// accumulators held in VGPRs.
#pragma once

#include "scan2d_bwd_kernels.hpp"
#include "scan2d_bwd_shared.hpp"
#include "scan2d_bwd_small.hpp"
#include "scan2d_fwd_shared.hpp"

namespace scan2d {

#define SCAN2D_BWD_VARIANTS(X)                                             \
    X(16, 4, 1, 4, 4, true) X(16, 8, 1, 4, 4, true) X(16, 12, 1, 4, 4, false) X(16, 16, 1, 4, 2, true) \
    X(16, 4, 4, 4, 2, true) X(16, 8, 4, 4, 1, true)                                                   \
    X(64, 4, 2, 8, 4, false) X(64, 8, 2, 8, 2, false) X(64, 16, 4, 4, 1, false)                           \
    X(64, 4, 4, 16, 2, false) X(64, 8, 4, 16, 1, false) X(64, 4, 1, 16, 2, false)

using BwdKernel = void (*)(const BwdArgs);
struct BwdKernels {
    BwdKernel ckpt = nullptr; BwdKernel main = nullptr; int RB = 0; int ckpt_NW = 0;
    int ckpt_LG = 0, ckpt_waves = 0;      // the checkpoint sweep may use another lane tiling than the main sweep
    bool ckpt_fast = true;                // W is a multiple of the checkpoint sweep's columns per lane
    bool shared = false;                  // main sweep of scan2d_bwd_shared.hpp
    BwdKernel main_panels = nullptr;      // its instantiation that takes column panels (wave-wide tiling of two states per lane)
    BwdKernel main_gate = nullptr;        // its instantiation with the output gate's backward inside (softplus step, rows first)
    // checkpoint sweep run by the shared-producer forward kernel in its checkpoint mode (FwdArgs), with its tiling
    void (*ckpt_fwd)(const FwdArgs) = nullptr;
    int cf_LG = 0, cf_K = 0, cf_NW = 0, cf_NG = 0, cf_waves = 0, cf_RPB = 0;
    // the same tiling as a forward pass that also writes the checkpoints (training step: scan2d_fwd_saving)
    void (*train_fwd)(const FwdArgs) = nullptr;
};

// Main sweeps that share the per-position work of a job through LDS: (LG, K, NW, NG, WAVES, RB) and the tiling
// (LG, K, NW) of the checkpoint sweep that goes with them (same RB, 4 waves per workgroup for 16-lane groups,
// as many as the main sweep otherwise).  N = NG * NW exactly; K even; NG * LG a multiple of 64.
// The last six numbers: the tiling (LG, K, NW, NG, WAVES, RPB) of the shared-producer forward kernel that runs the
// checkpoint sweep in its checkpoint mode.
#define SCAN2D_BWD_SHARED_VARIANTS(X)                                                       \
    X(16, 4, 1, 16, 4, 4, 16, 4, 2, 16, 4, 2, 8, 4, 4) X(16, 8, 1, 16, 4, 4, 16, 8, 2, 16, 8, 2, 8, 4, 2)       \
    X(16, 12, 1, 16, 4, 4, 16, 12, 2, 16, 12, 2, 8, 4, 2) X(32, 6, 1, 16, 8, 2, 16, 12, 2, 16, 12, 2, 8, 4, 2)  \
    X(32, 4, 1, 16, 8, 4, 16, 8, 2, 16, 8, 2, 8, 4, 2) X(64, 4, 1, 16, 16, 2, 64, 4, 1, 64, 4, 2, 8, 8, 4) \
    X(64, 4, 2, 8, 8, 2, 64, 4, 2, 64, 4, 2, 8, 8, 4)

// W: the map width (the checkpoint sweep has its own columns per lane, hence its own row-end treatment)
BwdKernels bwd_shared_kernels_f32(int LG, int K, int NW, int NG, int waves, int W, bool sp);
BwdKernels bwd_shared_kernels_bf16(int LG, int K, int NW, int NG, int waves, int W, bool sp);
// The columns-first instantiations (16-lane tilings only; everything else runs columns first through transposes)
BwdKernels bwd_shared_kernels_f32_cf(int LG, int K, int NW, int NG, int waves, int W, bool sp);
BwdKernels bwd_shared_kernels_bf16_cf(int LG, int K, int NW, int NG, int waves, int W, bool sp);

template <typename T, bool SP, bool CF = false>
inline BwdKernels lookup_bwd_shared_kernels(int LG, int K, int NW, int NG, int waves, int W) {
    BwdKernels r;
#define SCAN2D_X(lg, k, nw, ng, wv, rb, clg, ck, cnw, flg, fk, fnw, fng, fwv, frpb)                      \
    if constexpr (!CF || lg == 16) {                                                                     \
    if (LG == lg && K == k && NW == nw && NG == ng && waves == wv) {                                     \
        constexpr int cwv = clg == 16 ? 4 : wv;                                                          \
        const bool fast = W % k == 0, cfast = W % ck == 0;                                               \
        r.ckpt = cfast ? scan2d_bwd_ckpt_kernel<T, clg, ck, cnw, cwv, rb, true, SP, false, CF>           \
                       : scan2d_bwd_ckpt_kernel<T, clg, ck, cnw, cwv, rb, false, SP, false, CF>;         \
        r.ckpt_NW = cnw; r.ckpt_LG = clg; r.ckpt_waves = cwv; r.ckpt_fast = cfast;                       \
        r.main = fast ? scan2d_bwd_shared_kernel<T, lg, k, nw, ng, wv, rb, true, SP, CF>                 \
                      : scan2d_bwd_shared_kernel<T, lg, k, nw, ng, wv, rb, false, SP, CF>;               \
        r.RB = rb; r.shared = true;                                                                      \
        if constexpr (SP && !CF)                                                                         \
            r.main_gate = fast ? scan2d_bwd_shared_kernel<T, lg, k, nw, ng, wv, rb, true, true, false, false, true>       \
                               : scan2d_bwd_shared_kernel<T, lg, k, nw, ng, wv, rb, false, true, false, false, true>;     \
        if constexpr (!CF && lg == 64 && k == 4 && nw == 2)                                              \
            r.main_panels = fast ? scan2d_bwd_shared_kernel<T, lg, k, nw, ng, wv, rb, true, SP, false, true>      \
                                 : scan2d_bwd_shared_kernel<T, lg, k, nw, ng, wv, rb, false, SP, false, true>;    \
        if constexpr (Elem<T>::kBytes == 2) {                                                            \
            r.ckpt_fwd = (W % 2) != 0 ? scan2d_fwd_shared_kernel<T, flg, fk, fnw, fng, fwv, frpb, SP, true, rb, CF>     \
                                      : scan2d_fwd_shared_kernel<T, flg, fk, fnw, fng, fwv, frpb, SP, false, rb, CF>;   \
        } else {                                                                                         \
            r.ckpt_fwd = scan2d_fwd_shared_kernel<T, flg, fk, fnw, fng, fwv, frpb, SP, false, rb, CF>;   \
        }                                                                                                \
        r.cf_LG = flg; r.cf_K = fk; r.cf_NW = fnw; r.cf_NG = fng; r.cf_waves = fwv; r.cf_RPB = frpb;     \
        if constexpr (!SP && !CF && lg == 16) {                                                          \
            if constexpr (Elem<T>::kBytes == 2) {                                                        \
                r.train_fwd = (W % 2) != 0 ? scan2d_fwd_shared_kernel<T, flg, fk, fnw, fng, fwv, frpb, false, true, rb, false, true>    \
                                           : scan2d_fwd_shared_kernel<T, flg, fk, fnw, fng, fwv, frpb, false, false, rb, false, true>;  \
            } else {                                                                                     \
                r.train_fwd = scan2d_fwd_shared_kernel<T, flg, fk, fnw, fng, fwv, frpb, false, false, rb, false, true>;                 \
            }                                                                                            \
        }                                                                                                \
    }                                                                                                    \
    }
    SCAN2D_BWD_SHARED_VARIANTS(SCAN2D_X)
#undef SCAN2D_X
    return r;
}

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
        r.ckpt_NW = cnw; r.ckpt_LG = lg; r.ckpt_waves = wv; r.ckpt_fast = fast;                         \
        r.main = fast ? scan2d_bwd_main_kernel<T, lg, k, nw, wv, rb, true, pf, SP> : scan2d_bwd_main_kernel<T, lg, k, nw, wv, rb, false, pf, SP>; \
        r.RB = rb;                                                                                      \
    }
    SCAN2D_BWD_VARIANTS(SCAN2D_X)
#undef SCAN2D_X
    return r;
}

// Independent decay of the column recurrence (AV): the two 256-column tilings that cover every shape through column
// panels (one state per lane up to 16 states, four beyond), an ablation mode rather than a tuned path.
BwdKernels bwd_kernels_av_f32(int NW, bool fast);
BwdKernels bwd_kernels_av_bf16(int NW, bool fast);

template <typename T>
inline BwdKernels lookup_bwd_kernels_av(int NW, bool fast) {
    BwdKernels r;
    r.RB = 2; r.ckpt_NW = NW; r.ckpt_LG = 64; r.ckpt_waves = 16; r.ckpt_fast = fast;
    if (NW == 1) {
        r.ckpt = fast ? scan2d_bwd_ckpt_kernel<T, 64, 4, 1, 16, 2, true, false, true> : scan2d_bwd_ckpt_kernel<T, 64, 4, 1, 16, 2, false, false, true>;
        r.main = fast ? scan2d_bwd_main_kernel<T, 64, 4, 1, 16, 2, true, false, false, true> : scan2d_bwd_main_kernel<T, 64, 4, 1, 16, 2, false, false, false, true>;
    } else if (NW == 4) {
        r.ckpt = fast ? scan2d_bwd_ckpt_kernel<T, 64, 4, 4, 16, 2, true, false, true> : scan2d_bwd_ckpt_kernel<T, 64, 4, 4, 16, 2, false, false, true>;
        r.main = fast ? scan2d_bwd_main_kernel<T, 64, 4, 4, 16, 2, true, false, false, true> : scan2d_bwd_main_kernel<T, 64, 4, 4, 16, 2, false, false, false, true>;
    }
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
