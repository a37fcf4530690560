// Forward 2D selective scan, the form for maps whose states are spread over many lane groups
// (2DMamba Eq. 3, Eq. 5, Eq. 6, y = C h + D x).
//
// Same decomposition as scan2d_fwd.hpp (a lane group of LG lanes owns LG*K columns, each lane K columns and
// NW states, NG = N / NW lane groups share a map and walk down its rows), with one difference that matters
// when NG is large: everything that depends on the position and the channel only - widening x and the step,
// the softplus of the step, the mask select, step * x and Dskip * x - is computed ONCE per map and handed to
// the lane groups through LDS.  In the plain form every lane group repeats that work, which costs
// 9 instructions per position and lane group, i.e. 4.5 of the 18.8 instructions per (position, channel,
// state) on a 256x256 map with two states per lane.
//
//   * rows are processed in batches of RPB rows between two workgroup barriers;
//   * while batch b is scanned, each thread of a map produces RPB*K/NG cells of batch b+1: it reads their
//     x, step and mask bytes (requested one batch earlier), and writes step and step*x_eff as fp32 into the
//     LDS buffer of batch b+1; Dskip*x_eff stays in the thread's registers, because the same thread adds up
//     the partial sums of exactly those cells after the barrier of batch b+1;
//   * a scanning lane reads its K steps and K products of a row with 128-bit LDS loads one row ahead (no
//     vector-ALU slot), and Bm/Cm from a ring of raw registers as in the plain form;
//   * partial sums over states go to LDS; after the barrier every thread adds the NG partial sums of its
//     cells in index order (bit-reproducible), adds the skip term, rounds once and stores.
// LDS rows are stored chunk-wise ([K/4][LG][4] floats) so that the 128-bit accesses of neighbouring lanes
// fall into neighbouring banks for every K.
// Single-panel maps only (W <= LG*K) and N = NG*NW exactly; other shapes take the plain form.
#pragma once

#include "scan2d_fwd.hpp"

namespace scan2d {

template <int LG, int K>
__device__ __forceinline__ int lds_col(int c) {          // column of a panel -> float index in an LDS row
    return ((c % K) / 4) * (LG * 4) + (c / K) * 4 + (c % 4);
}

// h[j] += pl[j] * H(lane to the left) for the lane's first K-1 columns: the carry of the row scan applied with
// the lane movement inside the multiply-add (no copy of the neighbour's state into a register of its own).
// The group's first lane has no source lane and is not written: its carry is 0.
#ifndef SCAN2D_DPP_APPLY
#define SCAN2D_DPP_APPLY 0
#endif
constexpr bool kDppApply = SCAN2D_DPP_APPLY != 0;

template <int LG, int K>
__device__ __forceinline__ void carry_apply(float* hl, const float* pl, const float& Hh) {
    static_assert(LG == 16 || LG == 64, "half-wave groups need the first lane of the upper half excluded");
#pragma unroll
    for (int j = 0; j < K - 1; ++j) {
        if constexpr (LG == 64) {
            if (j == 0) asm volatile("s_nop 1\n\tv_fmac_f32_dpp %0, %1, %2 wave_shr:1 row_mask:0xf bank_mask:0xf" : "+v"(hl[j]) : "v"(Hh), "v"(pl[j]));
            else asm volatile("v_fmac_f32_dpp %0, %1, %2 wave_shr:1 row_mask:0xf bank_mask:0xf" : "+v"(hl[j]) : "v"(Hh), "v"(pl[j]));
        } else {
            if (j == 0) asm volatile("s_nop 1\n\tv_fmac_f32_dpp %0, %1, %2 row_shr:1 row_mask:0xf bank_mask:0xf" : "+v"(hl[j]) : "v"(Hh), "v"(pl[j]));
            else asm volatile("v_fmac_f32_dpp %0, %1, %2 row_shr:1 row_mask:0xf bank_mask:0xf" : "+v"(hl[j]) : "v"(Hh), "v"(pl[j]));
        }
    }
}

// UA (bf16 only): rows of odd width; Bm/Cm rows then start on odd 2-byte boundaries every other row and
// are shifted into place where they are unpacked, as in the plain form.
// CK > 0: the checkpoint sweep of the backward pass instead of the forward pass.  The recurrences are the same;
// Cm, the sum over states and y are left out, and the column state h at the bottom of every band of CK rows is
// written to p.ck ([maps][p.nb][N][W], the state entering band (i+1)/CK after row i; the last row's is never needed).
// CF: columns first.  The column recurrence runs on u (v = a * v[i-1,j] + u, the register that persists from row to
// row), the row scan then runs on its result (h = a * h[i,j-1] + v) and y reads the scanned value: the same
// instructions in the other order.  The checkpoint sweep (CK > 0) then keeps v and needs no row scan at all.
// KEEPY (with CK > 0): the forward pass of a training step - y is produced as usual and the band checkpoints are written
// on the way, so that the backward pass need not run its checkpoint sweep.
// GATE: the output gate of the block (Fig. 2) in the same kernel: the thread that produces a cell also loads z there,
// keeps SiLU(z) beside the skip term, and multiplies the unrounded sum over states by it where it stores the cell
// (p.y_gated; the ungated p.y is stored too unless it is null).
// SKEW: the row recurrence without a scan across the lanes.  Lane l of a 16-lane group works on row t - l at step t
// (H + 15 steps instead of H), so the state its row recurrence starts from is the last local state of the lane to its
// left at the previous step: one multiply-add with a DPP source replaces the decay prefix, the log-step scan and the
// carry multiply-add.  The LDS buffers keep their layout (a "row" of a batch is a step: the cell of step t and lane
// l belongs to row t - l); what changes are the global addresses of the producers' loads, of the Bm / Cm loads and
// of the stores, which follow the diagonal.  Cells of rows outside the map are produced as step = 0, x = 0 (decay 1,
// input 0: the column state stays 0 above the map) and never stored.  One state per lane, rows first, forward only.
// A measured alternative, reachable only through the tuning override: the dispatcher never ranks it.  On 256 maps of
// 256x256 bf16 positions it needs 11-12 vector instructions per (position, channel, state) against 15.4, but every
// access to memory follows the diagonal in pieces of one lane's K columns, and with 16 columns per lane a compute unit
// holds one wavefront per SIMD: 309 us (16 lanes x 16 columns) and 658 us (64 lanes x 4 columns) against 125 us.
template <typename T, int LG, int K, int NW, int NG, int WAVES, int RPB, bool SP, bool UA, int CK = 0, bool CF = false, bool KEEPY = false,
          bool GATE = false, bool SKEW = false>
__global__ __launch_bounds__(WAVES * 64) void scan2d_fwd_shared_kernel(const FwdArgs p) {
    static_assert(!SKEW || ((LG == 16 || LG == 64) && NW == 1 && CK == 0 && !CF && !UA), "skewed rows: 16- or 64-lane groups, one state per lane, forward, rows first");
    constexpr bool YOUT = CK == 0 || KEEPY;               // Cm, the sum over states and y are part of this instantiation
    constexpr bool NOSCAN = CF && CK > 0 && !KEEPY;       // columns-first checkpoint sweep: the row scan feeds nothing
    static_assert(!UA || Elem<T>::kBytes == 2, "UA: bf16 rows on odd 2-byte boundaries");
    constexpr int XW = words_of<T, K>();
    constexpr int SLOTS = WAVES * 64 / LG, MPW = SLOTS / NG, PANEL = LG * K, TM = NG * LG;
    static_assert(SLOTS % NG == 0 && MPW >= 1, "whole maps per workgroup");
    constexpr int CT = RPB * K / NG;                       // cells of a batch per thread
    static_assert(CT * NG == RPB * K && CT >= 1, "cells per thread");
    static_assert(RPB % 2 == 0, "rows are read from LDS one ahead, two register sets");
    constexpr int VEC = CT % 4 == 0 ? 4 : (CT % 2 == 0 ? 2 : 1);
    constexpr int NV = CT / VEC, VPR = PANEL / VEC;
    constexpr int SC = (NW < 4 ? NW : (K >= 12 ? 2 : 4));
    static_assert(NW % SC == 0, "state chunking");
    constexpr int PP_ROW = 2 * PANEL, PP_MAP = RPB * PP_ROW, PP_BUF = MPW * PP_MAP;
    constexpr int YP_ROW = SLOTS * PANEL, YP_BUF = RPB * YP_ROW;
    extern __shared__ float smem[];
    float* const pp = smem;                                // [2][MPW][RPB][2][PANEL]: step, step * x_eff
    float* const ypart = smem + 2 * PP_BUF;                // [2][RPB][SLOTS][PANEL]: partial sums over states

    const int tid = threadIdx.x;
    const int slot = tid / LG, l = tid % LG;
    int map_local = slot / NG;
    const int sg = slot - map_local * NG;
    const int tm = sg * LG + l;                            // thread index inside the map
    const long long map0 = (long long)blockIdx.x * MPW;
    const bool live = map0 + map_local < p.maps;
    const int map_slot = map_local;                        // LDS region (idle groups keep their own)
    if (!live) map_local = 0;                              // idle group: valid addresses, no stores
    const long long map = map0 + map_local;

    const int H = p.H, W = p.W, N = p.N;
    const size_t HW = (size_t)H * W;
    const int b0 = (int)(map0 / p.Dc);
    const int b = (int)(map / p.Dc), c = (int)(map % p.Dc);
    const int n0 = sg * NW;

    const T* __restrict__ xu = reinterpret_cast<const T*>(p.x) + (size_t)map0 * HW;
    const T* __restrict__ du = reinterpret_cast<const T*>(p.delta) + (size_t)map0 * HW;
    T* __restrict__ yu = reinterpret_cast<T*>(p.y) + (size_t)map * HW;
    const T* __restrict__ zu = reinterpret_cast<const T*>(p.z) + (size_t)map0 * HW;                // GATE only
    T* __restrict__ ygu = reinterpret_cast<T*>(p.y_gated) + (size_t)map * HW;                        // GATE only
    const T* __restrict__ Bu = reinterpret_cast<const T*>(p.Bm) + (size_t)b0 * N * HW;
    const T* __restrict__ Cu = reinterpret_cast<const T*>(p.Cm) + (size_t)b0 * N * HW;
    const uint8_t* __restrict__ mu = p.mask ? p.mask + (size_t)b0 * HW : nullptr;
    const uint32_t xlane = (uint32_t)(map_local * HW);
    const uint32_t slane = (uint32_t)(((size_t)(b - b0) * N + n0) * HW);
    const uint32_t mlane = (uint32_t)((size_t)(b - b0) * HW);
    constexpr uint32_t EB = (uint32_t)Elem<T>::kBytes;
    const size_t left_maps = (size_t)(p.maps - map0) * HW, left_items = (size_t)(p.maps / p.Dc - b0) * HW;
    auto up4 = [](size_t bytes) { return (bytes + 3) & ~(size_t)3; };
    const rsrc_t rsx = make_rsrc(xu, up4(left_maps * EB)), rsd = make_rsrc(du, up4(left_maps * EB)),
                 rsB = make_rsrc(Bu, up4(left_items * N * EB)), rsC = make_rsrc(Cu, up4(left_items * N * EB)),
                 rsm = make_rsrc(mu, up4(left_items));
    const rsrc_t rsz = make_rsrc(GATE ? zu : xu, up4(left_maps * EB));

    float Ap[NW];
#pragma unroll
    for (int s = 0; s < NW; ++s) Ap[s] = p.A[(size_t)c * N + n0 + s] * kLog2e;   // a = exp2(step * A * log2 e)
    const float dsk = p.Dskip != nullptr ? p.Dskip[c] : 0.0f;
    const float dbias = (SP && p.delta_bias != nullptr) ? p.delta_bias[c] : 0.0f;
    const bool has_mask = mu != nullptr;

    // ---- the cells this thread produces and later sums: vector v covers VEC columns of one row of a batch
    uint32_t cell_off[NV];     // element offset of the vector inside the batch (row * W + column)
    int cell_row[NV], cell_col[NV], cell_step[NV];
    static_assert(!SKEW || K % VEC == 0, "a vector of cells stays inside one lane's columns");
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int id = tm + v * TM;
        cell_row[v] = id / VPR;
        cell_col[v] = (id - cell_row[v] * VPR) * VEC;
        cell_off[v] = (uint32_t)cell_row[v] * (uint32_t)W + (uint32_t)cell_col[v];
        cell_step[v] = cell_row[v];                              // LDS row of the cell inside a batch
        if constexpr (SKEW) cell_row[v] -= cell_col[v] / K;      // map row of the cell relative to the batch's first step
    }
    const int nsteps = SKEW ? H + LG - 1 : H;
    const int nbatch = (nsteps + RPB - 1) / RPB;
    auto clamp_row = [&](int i) { return min(max(i, 0), H - 1); };

    uint32_t rawx[CT], rawd[CT], rawm[CT], rawz[GATE ? CT : 1];
    // element loads: any alignment, any width; a load past the end of the tensor returns 0
    auto request = [&](int batch) {
        const uint32_t ro = SKEW ? 0u : (uint32_t)batch * (uint32_t)(RPB * W);
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            if constexpr (SKEW)          // the cell's own row (clamped into the map: cells outside are produced as zeros)
                cell_off[v] = (uint32_t)clamp_row(batch * RPB + cell_row[v]) * (uint32_t)W + (uint32_t)cell_col[v];
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const uint32_t lo = xlane + cell_off[v] + (uint32_t)e;
                if constexpr (EB == 4) {
                    rawx[v * VEC + e] = __builtin_amdgcn_raw_buffer_load_b32(rsx, lo * 4u, ro * 4u, 0);
                    rawd[v * VEC + e] = __builtin_amdgcn_raw_buffer_load_b32(rsd, lo * 4u, ro * 4u, 0);
                    if constexpr (GATE) rawz[v * VEC + e] = __builtin_amdgcn_raw_buffer_load_b32(rsz, lo * 4u, ro * 4u, 0);
                } else {
                    rawx[v * VEC + e] = (uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rsx, lo * 2u, ro * 2u, 0);
                    rawd[v * VEC + e] = (uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rsd, lo * 2u, ro * 2u, 0);
                    if constexpr (GATE) rawz[v * VEC + e] = (uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rsz, lo * 2u, ro * 2u, 0);
                }
                rawm[v * VEC + e] = 0u;
                if (has_mask)
                    rawm[v * VEC + e] = (uint32_t)(uint8_t)__builtin_amdgcn_raw_buffer_load_b8(rsm, mlane + cell_off[v] + (uint32_t)e, ro, 0);
            }
        }
    };
    float sk_cur[CT], sk_next[CT], gt_cur[GATE ? CT : 1], gt_next[GATE ? CT : 1];
    auto produce = [&](int buf, int batch) {
        float* base = pp + buf * PP_BUF + map_slot * PP_MAP;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            float* row = base + cell_step[v] * PP_ROW + lds_col<LG, K>(cell_col[v]);
            const bool inside = !SKEW || (unsigned)(batch * RPB + cell_row[v]) < (unsigned)H;
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const int k = v * VEC + e;
                float dl = EB == 4 ? __uint_as_float(rawd[k]) : __uint_as_float(rawd[k] << 16);
                if constexpr (SP) dl = softplus_f32(dl + dbias);
                if constexpr (SKEW) dl = inside ? dl : 0.0f;
                const float xv = EB == 4 ? __uint_as_float(rawx[k]) : __uint_as_float(rawx[k] << 16);
                const float xe = (rawm[k] != 0u || !inside) ? 0.0f : xv;     // select: nothing under the mask leaks
                row[e] = dl;
                row[PANEL + e] = dl * xe;
                sk_next[k] = dsk * xe;
                if constexpr (GATE) {
                    const float zv = EB == 4 ? __uint_as_float(rawz[k]) : __uint_as_float(rawz[k] << 16);
                    gt_next[k] = zv * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-zv * kLog2e));  // SiLU(z)
                }
            }
        }
    };

    // ---- Bm / Cm: ring of raw registers, PDS rows ahead
    constexpr int XWR = XW + (UA ? 1 : 0);
    constexpr int SSET = 2 * NW * XWR;
    constexpr int PDS = (4 * SSET <= kPrefetchBudgetS && RPB % 4 == 0) ? 4 : (2 * SSET <= kPrefetchBudgetS ? 2 : 1);
    const int col0 = l * K;
    const uint32_t lcol = col0 < W ? (uint32_t)col0 : 0u;      // lanes past the last column mirror lane 0
    uint32_t rB[PDS][NW][XWR], rC[PDS][NW][XWR];
    auto lds = [&](rsrc_t rs, int s, uint32_t row_off, uint32_t* r) {
        if constexpr (SKEW) {          // row_off differs from lane to lane: it is part of the vector offset
            buffer_load_words<XW>(rs, (slane + lcol + row_off) * EB, (uint32_t)s * (uint32_t)HW * EB, r);
            return;
        }
        const uint32_t uni = (uint32_t)s * (uint32_t)HW + row_off;
        if constexpr (UA) buffer_load_words<XWR>(rs, ((slane + lcol + uni) * EB) & ~3u, 0u, r);   // rounded down to a dword
        else buffer_load_words<XW>(rs, (slane + lcol) * EB, uni * EB, r);
    };
    auto unpacks = [&](const uint32_t* raw, int s, uint32_t row_off, uint32_t* out) {
        if constexpr (UA) {
            const uint32_t uni = (uint32_t)s * (uint32_t)HW + row_off;
            const uint32_t sh = ((uni ^ (slane + lcol)) & 1u) << 4;
#pragma unroll
            for (int w = 0; w < XW; ++w) out[w] = __builtin_amdgcn_alignbit(raw[w + 1], raw[w], sh);
        } else {
#pragma unroll
            for (int w = 0; w < XW; ++w) out[w] = raw[w];
        }
    };

    float h[NW][K];
#pragma unroll
    for (int s = 0; s < NW; ++s)
#pragma unroll
        for (int j = 0; j < K; ++j) h[s][j] = 0.0f;            // h[-1, j] = 0
    float hrow[NW];                                            // SKEW: row state at this lane's last column, previous step
#pragma unroll
    for (int s = 0; s < NW; ++s) hrow[s] = 0.0f;

    // ---- prologue: batch 0 into LDS, batch 1 requested, first rows of Bm / Cm in flight
    request(0);
#pragma unroll
    for (int d = 0; d < PDS; ++d) {
        const uint32_t ro = (uint32_t)clamp_row(d - (SKEW ? l : 0)) * (uint32_t)W;
#pragma unroll
        for (int s = 0; s < NW; ++s) {
            lds(rsB, s, ro, rB[d][s]);
            if constexpr (YOUT) lds(rsC, s, ro, rC[d][s]);
        }
    }
    produce(0, 0);
#pragma unroll
    for (int k = 0; k < CT; ++k) {
        sk_cur[k] = sk_next[k];
        if constexpr (GATE) gt_cur[k] = gt_next[k];
    }
    request(min(1, nbatch - 1));
    __syncthreads();

    float dlq[2][K], dxq[2][K];
    auto fetch_row = [&](int buf, int r, int set) {
        const float* row = pp + buf * PP_BUF + map_slot * PP_MAP + r * PP_ROW + l * 4;
#pragma unroll
        for (int j4 = 0; j4 < K / 4; ++j4) {
            const float4 a = *reinterpret_cast<const float4*>(row + j4 * (LG * 4));
            const float4 d = *reinterpret_cast<const float4*>(row + PANEL + j4 * (LG * 4));
            dlq[set][4 * j4] = a.x; dlq[set][4 * j4 + 1] = a.y; dlq[set][4 * j4 + 2] = a.z; dlq[set][4 * j4 + 3] = a.w;
            dxq[set][4 * j4] = d.x; dxq[set][4 * j4 + 1] = d.y; dxq[set][4 * j4 + 2] = d.z; dxq[set][4 * j4 + 3] = d.w;
        }
    };
    fetch_row(0, 0, 0);

    for (int bt = 0; bt < nbatch; ++bt) {
        const int buf = bt & 1;
        const int row0 = bt * RPB;
#pragma unroll
        for (int r = 0; r < RPB; ++r) {
            const int i = row0 + r;
            const int set = r & 1, SS = r % PDS;
            if (r + 1 < RPB) fetch_row(buf, r + 1, set ^ 1);
            const uint32_t cur = (uint32_t)min(i, H - 1) * (uint32_t)W;                    // only the UA form reads it
            const uint32_t nxt = (uint32_t)(SKEW ? clamp_row(i + PDS - l) : min(i + PDS, H - 1)) * (uint32_t)W;
            float yacc[K];
#pragma unroll
            for (int s0 = 0; s0 < NW; s0 += SC) {
                float a[SC][K], hl[SC][K], pl[SC][K];
                float P[SC], Hh[SC], cin[SC];
#pragma unroll
                for (int t = 0; t < SC; ++t) {
                    const int s = s0 + t;
#pragma unroll
                    for (int j = 0; j < K; ++j) a[t][j] = __builtin_amdgcn_exp2f(dlq[set][j] * Ap[s]);
                    uint32_t uB[XW];
                    unpacks(rB[SS][s], s, cur, uB);
                    if constexpr (CF) {
#pragma unroll
                        for (int j = 0; j < K; ++j)      // column recurrence first; plain fmaf: a comes straight from v_exp_f32
                            h[s][j] = fmaf(a[t][j], h[s][j], dxq[set][j] * get_elem<T, K>(uB, j));
                        hl[t][0] = h[s][0];
                    } else {
                        hl[t][0] = dxq[set][0] * get_elem<T, K>(uB, 0);
                    }
                    if constexpr (SKEW) {
                        // Eq. 5 across the lane boundary: the row this lane works on was the left neighbour's row one
                        // step ago, and hrow holds the state that neighbour ended with.  The group's first lane has no
                        // source lane and is not written: its row starts from 0.
                        if constexpr (LG == 64)
                            asm volatile("s_nop 1\n\tv_fmac_f32_dpp %0, %1, %2 wave_shr:1 row_mask:0xf bank_mask:0xf"
                                         : "+v"(hl[t][0]) : "v"(hrow[s]), "v"(a[t][0]));
                        else
                            asm volatile("s_nop 1\n\tv_fmac_f32_dpp %0, %1, %2 row_shr:1 row_mask:0xf bank_mask:0xf"
                                         : "+v"(hl[t][0]) : "v"(hrow[s]), "v"(a[t][0]));
#pragma unroll
                        for (int j = 1; j < K; ++j) hl[t][j] = fmaf(a[t][j], hl[t][j - 1], dxq[set][j] * get_elem<T, K>(uB, j));
                        hrow[s] = hl[t][K - 1];
                        lds(rsB, s, nxt, rB[SS][s]);
                        continue;
                    }
                    pl[t][0] = a[t][0];
                    if constexpr (!NOSCAN) {
#pragma unroll
                        for (int j = 1; j < K; ++j) {
                            hl[t][j] = fmaf(a[t][j], hl[t][j - 1], CF ? h[s][j] : dxq[set][j] * get_elem<T, K>(uB, j));
                            pl[t][j] = pl[t][j - 1] * a[t][j];
                        }
                    }
                    // the refill of a ring slot stays behind the last use of the slot's old content (every instruction
                    // but a memory read may still cross): hoisted above it, the load needs a register pair of its own
                    // and the ring is rotated with copies at the end of every batch
                    __builtin_amdgcn_sched_barrier(0x7CF);
                    lds(rsB, s, nxt, rB[SS][s]);
                    if constexpr (!NOSCAN) {
                        P[t] = pl[t][K - 1];
                        Hh[t] = hl[t][K - 1];
                    }
                }
                if constexpr (!NOSCAN && !SKEW) {
                    if constexpr (kDppApply) group_scan_nocarry<LG, SC>(P, Hh, cin); else group_scan<LG, SC>(P, Hh, cin);
                }
#pragma unroll
                for (int t = 0; t < SC; ++t) {
                    const int s = s0 + t;
                    if constexpr (kDppApply && LG != 32 && !NOSCAN && !SKEW) carry_apply<LG, K>(hl[t], pl[t], Hh[t]);   // Eq. 5
                    uint32_t uC[XW];
                    if constexpr (YOUT) unpacks(rC[SS][s], s, cur, uC);
                    if constexpr (!NOSCAN) {
#pragma unroll
                        for (int j = 0; j < K; ++j) {
                            const float hh = SKEW ? hl[t][j]
                                           : (j == K - 1) ? Hh[t] : ((kDppApply && LG != 32) ? hl[t][j] : fmaf(pl[t][j], cin[t], hl[t][j]));
                            if constexpr (!CF) fma_inplace(h[s][j], a[t][j], hh);                   // Eq. 6
                            if constexpr (YOUT) {
                                const float cv = get_elem<T, K>(uC, j);
                                const float hv = CF ? hh : h[s][j];
                                yacc[j] = s == 0 ? cv * hv : fmaf(cv, hv, yacc[j]);
                            }
                        }
                    }
                    if constexpr (YOUT) lds(rsC, s, nxt, rC[SS][s]);
                }
            }
            if constexpr (YOUT) {
                float* mine = ypart + buf * YP_BUF + r * YP_ROW + slot * PANEL + l * 4;
#pragma unroll
                for (int j4 = 0; j4 < K / 4; ++j4)
                    *reinterpret_cast<float4*>(mine + j4 * (LG * 4)) =
                        make_float4(yacc[4 * j4], yacc[4 * j4 + 1], yacc[4 * j4 + 2], yacc[4 * j4 + 3]);
            }
            if constexpr (CK > 0) {
                if ((i + 1) % CK == 0 && i + 1 < H && live) {             // h[i] enters band (i+1)/CK
                    const int band = (i + 1) / CK;
#pragma unroll
                    for (int s = 0; s < NW; ++s) {
                        if (p.ck_chunked) {                            // every lane of the group writes, also past the last column
                            float* dst = p.ck + (((size_t)map * p.nb + band) * N + n0 + s) * PANEL + l * 4;
#pragma unroll
                            for (int j4 = 0; j4 < K / 4; ++j4)
                                *reinterpret_cast<float4*>(dst + j4 * (LG * 4)) =
                                    make_float4(h[s][4 * j4], h[s][4 * j4 + 1], h[s][4 * j4 + 2], h[s][4 * j4 + 3]);
                            continue;
                        }
                        float* dst = p.ck + (((size_t)map * p.nb + band) * N + n0 + s) * W + col0;
                        if (col0 + K <= W) {
                            uint32_t bits[K];
#pragma unroll
                            for (int j = 0; j < K; ++j) bits[j] = __float_as_uint(h[s][j]);
                            store_words<K>(reinterpret_cast<uint32_t*>(dst), bits);
                        } else {
#pragma unroll
                            for (int j = 0; j < K; ++j)
                                if (col0 + j < W) dst[j] = h[s][j];
                        }
                    }
                }
            }
        }
        // the next batch's cells: produced before the barrier (its LDS buffer was last read one batch ago,
        // before the previous barrier), then the loads of the batch after that are requested
        produce(buf ^ 1, bt + 1);
        request(min(bt + 2, nbatch - 1));
        __syncthreads();
        fetch_row(buf ^ 1, 0, 0);
        // sums over the lane groups of the cells this thread produced, skip term, one rounding, store
        if (YOUT && live) {
            const float* ybase = ypart + buf * YP_BUF + (slot - sg) * PANEL;
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const float* src = ybase + cell_step[v] * YP_ROW + lds_col<LG, K>(cell_col[v]);
                float acc[VEC];
                if constexpr (VEC == 4) {
                    float4 t0 = *reinterpret_cast<const float4*>(src);
                    acc[0] = t0.x; acc[1] = t0.y; acc[2] = t0.z; acc[3] = t0.w;
#pragma unroll
                    for (int g = 1; g < NG; ++g) {
                        const float4 t = *reinterpret_cast<const float4*>(src + g * PANEL);
                        acc[0] += t.x; acc[1] += t.y; acc[2] += t.z; acc[3] += t.w;
                    }
                } else if constexpr (VEC == 2) {
                    float2 t0 = *reinterpret_cast<const float2*>(src);
                    acc[0] = t0.x; acc[1] = t0.y;
#pragma unroll
                    for (int g = 1; g < NG; ++g) {
                        const float2 t = *reinterpret_cast<const float2*>(src + g * PANEL);
                        acc[0] += t.x; acc[1] += t.y;
                    }
                } else {
                    acc[0] = src[0];
#pragma unroll
                    for (int g = 1; g < NG; ++g) acc[0] += src[g * PANEL];
                }
                const int i = row0 + cell_row[v];
                if ((unsigned)i < (unsigned)H) {
                    float out[VEC];
#pragma unroll
                    for (int e = 0; e < VEC; ++e) out[e] = acc[e] + sk_cur[v * VEC + e];
                    auto store_vec = [&](T* base, const float* val) {
                        T* dst = base + (size_t)i * W + cell_col[v];
                        if (cell_col[v] + VEC <= W) {
                            if constexpr (EB == 4) {
                                uint32_t bits[VEC];
#pragma unroll
                                for (int e = 0; e < VEC; ++e) bits[e] = __float_as_uint(val[e]);
                                store_words<VEC>(reinterpret_cast<uint32_t*>(dst), bits);
                            } else if (VEC >= 2 && (((size_t)i * W + cell_col[v]) & 1u) == 0u) {   // pairs on dword boundaries
                                uint32_t bits[VEC >= 2 ? VEC / 2 : 1];
#pragma unroll
                                for (int e = 0; e < VEC / 2; ++e)
                                    bits[e] = f32_to_bf16_bits(val[2 * e]) | (f32_to_bf16_bits(val[2 * e + 1]) << 16);
                                store_words<(VEC >= 2 ? VEC / 2 : 1)>(reinterpret_cast<uint32_t*>(dst), bits);
                            } else {
#pragma unroll
                                for (int e = 0; e < VEC; ++e) store_elem(dst + e, val[e]);
                            }
                        } else {
#pragma unroll
                            for (int e = 0; e < VEC; ++e)
                                if (cell_col[v] + e < W) store_elem(dst + e, val[e]);
                        }
                    };
                    if constexpr (GATE) {
                        float gated[VEC];
#pragma unroll
                        for (int e = 0; e < VEC; ++e) gated[e] = out[e] * gt_cur[v * VEC + e];
                        store_vec(ygu, gated);
                        if (p.y != nullptr) store_vec(yu, out);
                    } else {
                        store_vec(yu, out);
                    }
                }
            }
        }
#pragma unroll
        for (int k = 0; k < CT; ++k) {
            sk_cur[k] = sk_next[k];
            if constexpr (GATE) gt_cur[k] = gt_next[k];
        }
    }
}

}  // namespace scan2d
