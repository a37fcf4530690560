// Backward main sweep, the form whose lane groups share the per-position work of a map through LDS
// (2DMamba Supp. B: two forward scans rebuild the states, a reverse column scan and a reverse row scan carry
// the gradients).  Same banded organisation as scan2d_bwd_main_kernel (scan2d_bwd_kernels.hpp): bands of RB
// rows walked bottom-up, per band and channel the states h[i-1,j] and hhor[i,j-1] are rebuilt into registers
// from the band's checkpoint, then the band's rows are walked upwards with g (reverse column recurrence, an
// FMA on a register that persists from row to row) and q (reverse row recurrence: serial over the lane's
// columns plus a leftward lane-group scan); dBm/dCm accumulate in registers over the GS channels of a
// workgroup; a*g of every channel waits in LDS between two bands.
//
// What differs: with one state per lane, the N lane groups of a map each repeated everything that depends on
// the position and the channel only - unpacking x, step, dy and the mask, the selects, step*x, Dskip*dy - in
// both passes over a band: 17 of the 55 instructions per (position, channel, state).  Here the threads of a
// job produce those values once per (band, channel) - each thread a few cells, loaded one (band, channel)
// ahead - and leave them in LDS as fp32:
//     dl = step       xe = mask ? 0 : x       dxe = dl * xe       dyv = dy       and the mask flag itself.
// The scanning lanes read their K columns with wide LDS loads; only Bm and Cm still come from global memory.
// The sums over the states of ddelta and dx go through LDS (double-buffered per row); the threads of the job add
// them up over the lane groups, add the skip term Dskip * dy and write +0 under the mask.  Where a row has more
// (column, tensor) pairs than the job has threads, the two sums are those of the decay gradients times a * A and of
// the gradients of u times B, one thread per column forms both and only then applies the factors that depend on the
// position alone (ddelta = first sum + x * second sum, dx = step * second sum): two instructions per state less.
// dA is summed over the lane group once per (band, channel) (DPP) and accumulated by one lane in LDS; dDskip
// is accumulated by the producing threads and summed per wavefront: both in a fixed order, so results are
// bit-reproducible.  K only has to be even here (the scanning lanes load no mask bytes), which allows
// half-wave groups of 6 columns on 192-wide maps: band state of 96 registers, two waves per SIMD.
// MP instantiations - column panels (maps wider than LG*K columns, one launch per panel, right to left; the other
// instantiations carry none of this code or its registers): p.cb is the panel's first column;
// the row-scan state entering from the left panel (p.hc_in, left by the checkpoint sweeps) starts lane 0's rebuilt
// row recurrence, a*q entering from the right panel (p.qc_in) joins the last lane's reverse recurrence, a*q of the
// panel's first column goes to p.qc_out, and dA / dDskip add to what the panels to the right have left (p.accum).
#pragma once

#include "scan2d_bwd_kernels.hpp"

namespace scan2d {

// Column of a panel -> float index in an LDS row stored chunk-wise: [K/4 chunks][LG][4], then [LG][K%4].
template <int LG, int K>
__device__ __forceinline__ int lds_colk(int c) {
    constexpr int K4 = (K / 4) * 4;
    const int j = c % K, l = c / K;
    return j < K4 ? (j / 4) * (LG * 4) + l * 4 + (j % 4) : (K4 / 4) * (LG * 4) + l * (K - K4) + (j - K4);
}
// The K values of lane l from such a row (128-bit loads, one 64-bit load for K % 4 == 2).
template <int LG, int K>
__device__ __forceinline__ void lds_read_k(const float* row, int l, float* out) {
    static_assert(K % 4 == 0 || K % 4 == 2, "columns per lane: even");
#pragma unroll
    for (int c4 = 0; c4 < K / 4; ++c4) {
        const float4 v = *reinterpret_cast<const float4*>(row + c4 * (LG * 4) + l * 4);
        out[4 * c4] = v.x; out[4 * c4 + 1] = v.y; out[4 * c4 + 2] = v.z; out[4 * c4 + 3] = v.w;
    }
    if constexpr (K % 4 == 2) {
        const float2 v = *reinterpret_cast<const float2*>(row + (K / 4) * (LG * 4) + l * 2);
        out[K - 2] = v.x; out[K - 1] = v.y;
    }
}
template <int LG, int K>
__device__ __forceinline__ void lds_write_k(float* row, int l, const float* v) {
#pragma unroll
    for (int c4 = 0; c4 < K / 4; ++c4)
        *reinterpret_cast<float4*>(row + c4 * (LG * 4) + l * 4) = make_float4(v[4 * c4], v[4 * c4 + 1], v[4 * c4 + 2], v[4 * c4 + 3]);
    if constexpr (K % 4 == 2) *reinterpret_cast<float2*>(row + (K / 4) * (LG * 4) + l * 2) = make_float2(v[K - 2], v[K - 1]);
}

// Sum over the LG lanes of a lane group; the group's last lane holds the total (LG = 16, 32 or 64).
template <int LG>
__device__ __forceinline__ float group_sum_last(float v) {
    asm volatile("s_nop 1\n\t"
                 "v_add_f32_dpp %0, %0, %0 row_shr:1 row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"
                 "v_add_f32_dpp %0, %0, %0 row_shr:2 row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"
                 "v_add_f32_dpp %0, %0, %0 row_shr:4 row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"
                 "v_add_f32_dpp %0, %0, %0 row_shr:8 row_mask:0xf bank_mask:0xf\n\ts_nop 1\n\t"
                 : "+v"(v));
    if constexpr (LG >= 32)
        asm volatile("v_add_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\ts_nop 1\n\t" : "+v"(v));
    if constexpr (LG == 64)
        asm volatile("v_add_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\ts_nop 1\n\t" : "+v"(v));
    return v;
}

// Mirror of a value inside its lane group (lane l <-> lane LG-1-l), through the LDS crossbar.
template <int LG>
__device__ __forceinline__ float group_mirror(float v) {
    const int lane = (int)(threadIdx.x & 63u);
    const int src = (lane & ~(LG - 1)) | (LG - 1 - (lane & (LG - 1)));
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(src << 2, __builtin_bit_cast(int, v)));
}
// Leftward scan of one recurrence over a lane group of any width (see group_scan_left): half-wave groups
// mirror the pair inside the group, scan rightwards and mirror the carry back.
template <int LG>
__device__ __forceinline__ void group_scan_left_any(float* P, float* Q, float* C) {
    if constexpr (LG == 32) {
        float Pm[1] = {group_mirror<32>(P[0])}, Qm[1] = {group_mirror<32>(Q[0])}, Cm[1];
        group_scan<32, 1>(Pm, Qm, Cm);
        C[0] = group_mirror<32>(Cm[0]);
    } else {
        group_scan_left<LG, 1>(P, Q, C);
    }
}
// Value held by the lane to the right inside the lane group (0 for the group's last lane).
template <int LG>
__device__ __forceinline__ float from_right_any(float v) {
    if constexpr (LG == 32) {
        const float r = from_right<64>(v);
        return (threadIdx.x & 31u) == 31u ? 0.0f : r;
    } else {
        return from_right<LG>(v);
    }
}

// Value held by the lane to the left inside the lane group (0 for the group's first lane).
template <int LG>
__device__ __forceinline__ float from_left_any(float v) {
    float r;
    if constexpr (LG == 16) {
        asm volatile("s_nop 1\n\tv_mov_b32_dpp %0, %1 row_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:0" : "=&v"(r) : "v"(v));
    } else {
        asm volatile("s_nop 1\n\tv_mov_b32_dpp %0, %1 wave_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:0" : "=&v"(r) : "v"(v));
        if constexpr (LG == 32) r = (threadIdx.x & 31u) == 0u ? 0.0f : r;
    }
    return r;
}

// d softplus(t) / dt from the softplus value itself: sp = log(1 + e^t), so the logistic function of t is 1 - e^(-sp).
// Below 1/64 the difference loses digits and the series takes over (next term: sp^4 / 24, under 2e-7 of the value).
__device__ __forceinline__ float dsoftplus_from_value(float sp) {
    const float big = 1.0f - __builtin_amdgcn_exp2f(-sp * kLog2e);
    const float small = sp * (1.0f - sp * (0.5f - sp * (1.0f / 6.0f)));
    return sp < 0.015625f ? small : big;
}

#ifndef SCAN2D_BWD_RECOMPUTE_HHOR
#define SCAN2D_BWD_RECOMPUTE_HHOR 1
#endif

// Dynamic LDS layout (floats), T = workgroup threads, SLOTS = T / LG, JPW = SLOTS / NG:
//   part [2][2][SLOTS][PANEL]      per-lane partial sums over its states of ddelta and dx (double buffered per row)
//   pp   [JPW][RB][5][PANEL]       the per-position values of the current (band, channel): dl, xe, dxe, dyv, mask flag
//   gaL  [GS][T][NW*K]             a[i+1,j]*g[i+1,j] of every channel, kept between bands
//   dAL  [GS][SLOTS][NW]           dA of every channel, accumulated over the bands
//   dDL  [GS][WAVES]               dDskip of every channel per wavefront, accumulated over the bands
//   dBL  [GS][WAVES]               (SPIN) the bias gradient, the sum of ddelta_raw, likewise
// CF: columns first (v = a * v[i-1,j] + u, then h = a * h[i,j-1] + v).  The checkpoints then hold v, the band
// arrays hold v[i-1,j] (in `hprev`) and h[i,j-1] (in `hhl`), the reverse row scan q runs on dy * Cm alone and the
// reverse column recurrence on its result (gv = q + a[i+1,j] * gv[i+1,j], kept in `ga` as a * gv); the gradient of u
// is gv, that of the decay gv * v[i-1,j] + q * h[i,j-1]: the same instructions in the other order.
// GATE: the backward of the block's output gate y = y_scan * SiLU(z) where the cells are produced: the thread that
// produces a cell also loads z and y_scan there, stores dz = dy * y_scan * s (1 + z (1 - s)), s the logistic function of
// z, and hands dy * SiLU(z), unrounded, to the sweeps in place of dy.
template <typename T, int LG, int K, int NW, int NG, int WAVES, int RB, bool FAST, bool SP, bool CF = false, bool MP = false, bool GATE = false>
__global__ __launch_bounds__(WAVES * 64) void scan2d_bwd_shared_kernel(const BwdArgs p) {
    static_assert(!MP || !CF, "column panels: rows first only");
    static_assert(!GATE || (SP && !MP), "the gate goes with the softplus step, single panel");
    // RECOMP: the row-scan states hhor[i,j-1] of a band are not kept from the rebuild to the reverse sweep (RB*NW*K
    // registers) but formed again there from the column states, which are kept anyway: Eq. 6 read backwards,
    // hhor[i,j] = h[i,j] - a[i,j] * h[i-1,j], one multiply-add per cell and one lane shift per row instead of a register
    // (in practice: a copy into and out of an accumulation register) per cell.  The difference to the kept value is one
    // rounding of h[i,j].
    constexpr bool RECOMP = SCAN2D_BWD_RECOMPUTE_HHOR != 0 && !CF && !MP;
    const int cb = MP ? p.cb : 0;                         // first column of this launch's panel
    constexpr int THREADS = WAVES * 64, SLOTS = THREADS / LG, JPW = SLOTS / NG, PANEL = LG * K, TMJ = NG * LG;
    static_assert(SLOTS % NG == 0 && JPW >= 1, "whole jobs per workgroup");
    constexpr int CELLS = RB * PANEL, CT = (CELLS + TMJ - 1) / TMJ;     // cells of a band per producing thread
    // Sums over the states of a row: where the job has fewer threads than (column, tensor) pairs, one thread per column
    // forms both sums and the factors that depend on the position alone (x, the step) are applied after them (LATEF);
    // otherwise one thread per (column, tensor) pair, the factors applied per state
    constexpr bool LATEF = 2 * PANEL > TMJ;
    constexpr int TASKS = LATEF ? PANEL : 2 * PANEL, TT = (TASKS + TMJ - 1) / TMJ;
    constexpr int XW = words_of<T, K>();
    // SP: p.delta is the raw projection.  Single-panel instantiations (SPIN) apply the softplus where the cells are
    // produced and the chain rule where ddelta is summed (the logistic factor comes from the step kept in LDS), so
    // ddelta receives the gradient of the raw projection directly; the column-panel instantiations read the step from a
    // buffer a kernel of its own has filled (fp32, p.delta) and write the step's gradient back over it.
    constexpr bool SPIN = SP && !MP;
    using DT = std::conditional_t<SP && !SPIN, float, T>;               // element type of what p.delta holds
    constexpr int PP_ROW = 5 * PANEL, PP_JOB = RB * PP_ROW;
    // Bm / Cm of the next row are requested before the current row is processed only where the registers allow it
    // (two waves per SIMD hide the latency otherwise)
#ifndef SCAN2D_BWD_SHARED_PF_LIMIT
#define SCAN2D_BWD_SHARED_PF_LIMIT 4
#endif
    constexpr bool PF = K * NW <= SCAN2D_BWD_SHARED_PF_LIMIT;
    constexpr int NB = PF ? 2 : 1;
    extern __shared__ float lds[];
    const int GS = p.GS;
    float* const part = lds;
    float* const pp = part + 4 * THREADS * K;
    float* const gaL = pp + JPW * PP_JOB;
    float* const dAL = gaL + (size_t)GS * THREADS * NW * K;
    float* const dDL = dAL + (size_t)GS * SLOTS * NW;
    float* const dBL = dDL + (size_t)GS * WAVES;             // SPIN instantiations only

    const int tid = threadIdx.x, slot = tid / LG, l = tid % LG, wave = tid / 64;
    int job_local = slot / NG;
    const int sg = slot - job_local * NG;
    const int tm = sg * LG + l;                           // thread index inside the job
    const long long jobs = (long long)p.Bt * p.CG;
    const long long job0 = (long long)blockIdx.x * JPW;
    const bool live = job0 + job_local < jobs;
    const int job_slot = job_local;
    if (!live) job_local = 0;
    const long long job = job0 + job_local;
    const int b = (int)(job / p.CG), cg = (int)(job % p.CG);
    const int c_first = cg * GS;
    const int nch = live ? min(GS, p.Dc - c_first) : 0;

    const int H = p.H, W = p.W, N = p.N;
    const size_t HW = (size_t)H * W;
    const int n0 = sg * NW;
    const int col0 = cb + l * K;                         // first column of this lane in the map
    const bool inside = col0 < W;
    const uint32_t lcol = inside ? (uint32_t)col0 : (uint32_t)cb;
    const TailRows<T> tl(p.tail, W);
    const bool lastm = b == p.Bt - 1;
    bool lastB[NW];
#pragma unroll
    for (int s = 0; s < NW; ++s) lastB[s] = lastm && (n0 + s == N - 1);
    const int nv = FAST ? (inside ? K : 0) : max(0, min(K, W - col0));   // cells of this lane inside the map
    const uint8_t* mm = p.mask ? p.mask + (size_t)b * HW : nullptr;
    const T* Bs[NW];
    const T* Cs[NW];
#pragma unroll
    for (int s = 0; s < NW; ++s) {
        Bs[s] = reinterpret_cast<const T*>(p.Bm) + ((size_t)b * N + n0 + s) * HW;
        Cs[s] = reinterpret_cast<const T*>(p.Cm) + ((size_t)b * N + n0 + s) * HW;
    }
    float* const ppj = pp + job_slot * PP_JOB;

    for (int ch = 0; ch < GS; ++ch) {
#pragma unroll
        for (int e = 0; e < NW * K; ++e) gaL[((size_t)ch * THREADS + tid) * (NW * K) + e] = 0.0f;   // g below the map is 0
        if (l == LG - 1) {
#pragma unroll
            for (int s = 0; s < NW; ++s) dAL[((size_t)ch * SLOTS + slot) * NW + s] = 0.0f;
        }
        if ((tid & 63) == 63) {
            dDL[ch * WAVES + wave] = 0.0f;
            if constexpr (SPIN) dBL[ch * WAVES + wave] = 0.0f;
        }
    }
    // gaL entries are private to a thread, dAL entries to the last lane of a lane group, dDL entries to the last
    // lane of a wavefront: no barrier needed for them until the final sums

    // ---- the cells this thread produces: index inside the band -> (row, column), fixed for the whole kernel
    int cell_r[CT], cell_c[CT];
    bool cell_ok[CT];
#pragma unroll
    for (int v = 0; v < CT; ++v) {
        const int id = tm + v * TMJ;
        cell_r[v] = id / PANEL;
        cell_c[v] = id - cell_r[v] * PANEL;
        cell_ok[v] = id < CELLS && live;
        if (!cell_ok[v]) { cell_r[v] = 0; cell_c[v] = 0; }
    }
    uint32_t rawx[CT], rawd[CT], rawy[CT], rawm[CT], rawz[GATE ? CT : 1], raws[GATE ? CT : 1];
    // Loads of the cells of (band, channel): clamped to a valid element, so that no load sits in a branch; what
    // lies outside the map is zeroed where the cell is produced.
    auto request = [&](int band, int ch) {
        const int c = c_first + min(ch, max(nch - 1, 0));
        const size_t map = (size_t)b * p.Dc + c;
        const T* xm = reinterpret_cast<const T*>(p.x) + map * HW;
        const DT* dm = reinterpret_cast<const DT*>(p.delta) + map * HW;
        const T* dym = reinterpret_cast<const T*>(p.dy) + map * HW;
        const T* zm = reinterpret_cast<const T*>(p.z) + map * HW;          // GATE only
        const T* ysm = reinterpret_cast<const T*>(p.y_scan) + map * HW;    // GATE only
#pragma unroll
        for (int v = 0; v < CT; ++v) {
            const int i = min(band * RB + cell_r[v], H - 1);
            const size_t o = (size_t)i * W + (size_t)min(cb + cell_c[v], W - 1);
            if constexpr (GATE) { rawz[v] = elem_bits(zm + o); raws[v] = elem_bits(ysm + o); }
            rawx[v] = elem_bits(xm + o);
            rawd[v] = elem_bits(dm + o);
            rawy[v] = elem_bits(dym + o);
            rawm[v] = mm != nullptr ? (uint32_t)mm[o] : 0u;
        }
    };
    auto widen = [](uint32_t bits, auto tag) -> float {
        using E = decltype(tag);
        if constexpr (Elem<E>::kBytes == 4) return __uint_as_float(bits);
        else return __uint_as_float(bits << 16);
    };

    int step = 0;                                         // rows reduced so far: parity picks the `part` buffer
    request(p.nb - 1, 0);
    for (int band = p.nb - 1; band >= 0; --band) {
        const int r0 = band * RB;
        const int ilast = min(r0 + RB, H) - 1;            // bottom row of the band
        float dBacc[RB][NW][K], dCacc[RB][NW][K];
#pragma unroll
        for (int r = 0; r < RB; ++r)
#pragma unroll
            for (int s = 0; s < NW; ++s)
#pragma unroll
                for (int j = 0; j < K; ++j) { dBacc[r][s][j] = 0.0f; dCacc[r][s][j] = 0.0f; }

        for (int ch = 0; ch < GS; ++ch) {
            const bool act = ch < nch;
            const int c = act ? c_first + ch : c_first;      // idle iterations re-read a valid channel
            const size_t map = (size_t)b * p.Dc + c;
            float* ddw = (SP && !SPIN) ? const_cast<float*>(reinterpret_cast<const float*>(p.delta)) + map * HW : nullptr;
            const float dbc = (SPIN && p.delta_bias != nullptr) ? p.delta_bias[c] : 0.0f;
            T* dxm = reinterpret_cast<T*>(p.dx) + map * HW;
            T* ddm = reinterpret_cast<T*>(p.ddelta) + map * HW;
            float An[NW], Ap[NW];
#pragma unroll
            for (int s = 0; s < NW; ++s) {
                An[s] = p.A[(size_t)c * N + n0 + s];
                Ap[s] = An[s] * kLog2e;
            }
            const float dsk = p.Dskip != nullptr ? p.Dskip[c] : 0.0f;

            // ---- the per-position values of this (band, channel).  The threads that sum the last row of the previous
            // (band, channel) still read its dy and mask flags: wait for them
            __syncthreads();
            float dDb = 0.0f, dBb = 0.0f;                      // dBb (SPIN): sum of the ddelta_raw this thread stores
#pragma unroll
            for (int v = 0; v < CT; ++v) {
                const bool in = cell_ok[v] && act && r0 + cell_r[v] < H && cb + cell_c[v] < W;
                const bool m = rawm[v] != 0u;
                float dl = widen(rawd[v], DT{});
                if constexpr (SPIN) dl = softplus_f32(dl + dbc);
                dl = in ? dl : 0.0f;
                const float xv = widen(rawx[v], T{});
                const float xe = (in && !m) ? xv : 0.0f;                 // select: nothing under the mask leaks
                float dyv = in ? widen(rawy[v], T{}) : 0.0f;
                if constexpr (GATE) {
                    const float zv = widen(rawz[v], T{}), sg = logistic_f32(zv);
                    if (in) store_elem(reinterpret_cast<T*>(p.dz) + map * HW + (size_t)(r0 + cell_r[v]) * W + (size_t)(cb + cell_c[v]),
                                       dyv * widen(raws[v], T{}) * (sg * fmaf(zv, 1.0f - sg, 1.0f)));
                    dyv *= zv * sg;
                }
                if (cell_ok[v]) {
                    float* row = ppj + cell_r[v] * PP_ROW + lds_colk<LG, K>(cell_c[v]);
                    row[0] = dl;
                    row[PANEL] = xe;
                    row[2 * PANEL] = dl * xe;
                    row[3 * PANEL] = dyv;
                    row[4 * PANEL] = m ? 1.0f : 0.0f;
                }
                dDb = fmaf(dyv, xe, dDb);
            }
            // the cells of the next (band, channel)
            if (ch + 1 < GS) request(band, ch + 1);
            else request(max(band - 1, 0), 0);
            __syncthreads();

            // ---- scans 1 and 2: rebuild h[i-1,j] and hhor[i,j-1] for the rows of the band
            float hprev[RB][NW][K], hhl[RECOMP ? 1 : RB][NW][K];
            float hcur[NW][K];                                 // after scans 1 and 2: the state of the band's bottom row
            {
                uint32_t fB[NB][NW][XW];
                auto issue = [&](int buf, int i) {
                    const size_t ro = (size_t)i * W;
                    const bool bottom = i == H - 1;
#pragma unroll
                    for (int s = 0; s < NW; ++s) ld_elems<T, K, FAST>(Bs[s] + ro, lcol, lastB[s] && bottom, tl.B, fB[buf][s]);
                };
                if constexpr (PF) issue(0, r0);
#pragma unroll
                for (int s = 0; s < NW; ++s) {
                    const float* src = p.ck + ((map * p.nb + band) * N + n0 + s) * W;
                    if (band == 0) {
#pragma unroll
                        for (int j = 0; j < K; ++j) hcur[s][j] = 0.0f;
                    } else {
                        if (p.ck_chunked) {
                            const float* cs = p.ck + ((map * p.nb + band) * N + n0 + s) * PANEL + l * 4;
#pragma unroll
                            for (int j4 = 0; j4 < K / 4; ++j4) {
                                const float4 v = *reinterpret_cast<const float4*>(cs + j4 * (LG * 4));
                                hcur[s][4 * j4] = v.x; hcur[s][4 * j4 + 1] = v.y; hcur[s][4 * j4 + 2] = v.z; hcur[s][4 * j4 + 3] = v.w;
                            }
                        } else {
                            load_f32s<K>(src + lcol, hcur[s]);           // past the row end: the next checkpoint row or the region behind
                        }
                        if constexpr (!FAST) {
#pragma unroll
                            for (int j = 0; j < K; ++j)
                                if (j >= nv) hcur[s][j] = 0.0f;
                        }
                    }
                }
#pragma unroll
                for (int r = 0; r < RB; ++r) {
                    const int i = r0 + r;
                    if (i < H) {
                        if constexpr (PF) { if (r + 1 < RB && i + 1 < H) issue((r + 1) & 1, i + 1); }
                        else issue(0, i);
                        float dl[K], dxe[K];
                        lds_read_k<LG, K>(ppj + r * PP_ROW, l, dl);
                        lds_read_k<LG, K>(ppj + r * PP_ROW + 2 * PANEL, l, dxe);
#pragma unroll
                        for (int s = 0; s < NW; ++s) {
                            float a[K], hl[K], pl[K];
#pragma unroll
                            for (int j = 0; j < K; ++j) a[j] = __builtin_amdgcn_exp2f(dl[j] * Ap[s]);
                            if constexpr (CF) {
#pragma unroll
                                for (int j = 0; j < K; ++j) {
                                    hprev[r][s][j] = hcur[s][j];                                   // v[i-1,j]
                                    hcur[s][j] = fmaf(a[j], hcur[s][j], dxe[j] * get_elem<T, K>(fB[PF ? (r & 1) : 0][s], j));
                                }
                                hl[0] = hcur[s][0];
                            } else {
                                hl[0] = dxe[0] * get_elem<T, K>(fB[PF ? (r & 1) : 0][s], 0);
                            }
                            float hcv = 0.0f;                             // state entering from the panel to the left
                            if constexpr (MP) {
                                if (p.hc_in != nullptr && l == 0) {
                                    hcv = p.hc_in[(map * N + n0 + s) * H + i];
                                    hl[0] = fmaf(a[0], hcv, hl[0]);
                                }
                            }
                            pl[0] = a[0];
#pragma unroll
                            for (int j = 1; j < K; ++j) {
                                hl[j] = fmaf(a[j], hl[j - 1], CF ? hcur[s][j] : dxe[j] * get_elem<T, K>(fB[PF ? (r & 1) : 0][s], j));
                                pl[j] = pl[j - 1] * a[j];
                            }
                            float P[1] = {pl[K - 1]}, Hh[1] = {hl[K - 1]}, cin[1];
                            group_scan<LG, 1>(P, Hh, cin);
                            float left = cin[0];                          // hhor[i, j-1] (CF: h[i, j-1])
                            if constexpr (MP) {
                                if (p.hc_in != nullptr && l == 0) left = hcv;
                            }
#pragma unroll
                            for (int j = 0; j < K; ++j) {
                                const float hh = (j == K - 1) ? Hh[0] : fmaf(pl[j], cin[0], hl[j]);
                                if constexpr (!RECOMP) hhl[r][s][j] = left;
                                if constexpr (!CF) {
                                    hprev[r][s][j] = hcur[s][j];
                                    hcur[s][j] = fmaf(a[j], hcur[s][j], hh);
                                }
                                left = hh;
                            }
                        }
                    } else if constexpr (!CF) {                  // below the map: the row above finds the bottom state here
#pragma unroll
                        for (int s = 0; s < NW; ++s)
#pragma unroll
                            for (int j = 0; j < K; ++j) hprev[r][s][j] = hcur[s][j];
                    }
                }
            }

            // ---- scans 3 and 4, bottom row of the band first
            float ga[NW][K], dAb[NW];
#pragma unroll
            for (int s = 0; s < NW; ++s) {
                dAb[s] = 0.0f;
#pragma unroll
                for (int j = 0; j < K; ++j) ga[s][j] = gaL[((size_t)ch * THREADS + tid) * (NW * K) + s * K + j];
            }
            uint32_t bB[NB][NW][XW], bC[NB][NW][XW];
            auto issue_r = [&](int buf, int i) {
                const size_t ro = (size_t)i * W;
                const bool bottom = i == H - 1;
#pragma unroll
                for (int s = 0; s < NW; ++s) {
                    ld_elems<T, K, FAST>(Bs[s] + ro, lcol, lastB[s] && bottom, tl.B, bB[buf][s]);
                    ld_elems<T, K, FAST>(Cs[s] + ro, lcol, lastB[s] && bottom, tl.C, bC[buf][s]);
                }
            };
#pragma unroll
            for (int r = RB - 1; r >= 0; --r) {
                const int i = r0 + r;
                if (i < H) {                                               // uniform over the workgroup
                    if constexpr (PF) {
                        if (i == ilast) issue_r(r & 1, i);
                        if (r > 0) issue_r((r - 1) & 1, i - 1);
                    } else {
                        issue_r(0, i);
                    }
                    const size_t ro = (size_t)i * W;
                    const float* prow = ppj + r * PP_ROW;
                    // ddl: sum over this lane's states of (gradient of the decay) * a * A; dxl: of (gradient of u) * B.  The
                    // factors that depend on the position only (x and the step) are applied after the sum over all states
                    float dl[K], xe[LATEF ? 1 : K], dxe[K], dyv[K], ddl[K], dxl[K];
                    lds_read_k<LG, K>(prow, l, dl);
                    if constexpr (!LATEF) lds_read_k<LG, K>(prow + PANEL, l, xe);
                    lds_read_k<LG, K>(prow + 2 * PANEL, l, dxe);
                    lds_read_k<LG, K>(prow + 3 * PANEL, l, dyv);
#pragma unroll
                    for (int j = 0; j < K; ++j) { ddl[j] = 0.0f; dxl[j] = 0.0f; }
#pragma unroll
                    for (int s = 0; s < NW; ++s) {
                        float a[K], Bv[K], g[K], hrow[RECOMP ? K : 1];
#pragma unroll
                        for (int j = 0; j < K; ++j) {
                            a[j] = __builtin_amdgcn_exp2f(dl[j] * Ap[s]);
                            Bv[j] = get_elem<T, K>(bB[PF ? (r & 1) : 0][s], j);
                            float hv;
                            if constexpr (CF) {                // v[i,j], then h[i,j]
                                const float hh = fmaf(a[j], hprev[r][s][j], dxe[j] * Bv[j]);
                                hv = fmaf(a[j], hhl[r][s][j], hh);
                            } else {                           // h[i,j] is what the row below started from
                                hv = r == RB - 1 ? hcur[s][j] : hprev[r + 1 < RB ? r + 1 : r][s][j];
                            }
                            dCacc[r][s][j] = fmaf(dyv[j], hv, dCacc[r][s][j]);
                            if constexpr (RECOMP) hrow[j] = fmaf(-a[j], hprev[r][s][j], hv);           // hhor[i,j]
                            const float dyC = dyv[j] * get_elem<T, K>(bC[PF ? (r & 1) : 0][s], j);
                            if constexpr (CF) {
                                g[j] = dyC;
                            } else {
                                g[j] = dyC + ga[s][j];                                                  // scan 3
                                ga[s][j] = a[j] * g[j];
                            }
                        }
                        if constexpr (RECOMP) {                  // hhor[i,j-1]: the left neighbour's last column for j = 0
                            hhl[0][s][0] = from_left_any<LG>(hrow[K - 1]);
#pragma unroll
                            for (int j = 1; j < K; ++j) hhl[0][s][j] = hrow[j - 1];
                        }
                        // scan 4: q[j] = g[j] + a[j+1] * q[j+1]
                        float ar[K], ql[K], pr[K];
#pragma unroll
                        for (int j = 0; j + 1 < K; ++j) ar[j] = a[j + 1];
                        ar[K - 1] = from_right_any<LG>(a[0]);
                        ql[K - 1] = g[K - 1];
                        if constexpr (MP) {
                            if (p.qc_in != nullptr && l == LG - 1)        // a*q entering from the panel to the right
                                ql[K - 1] += p.qc_in[(map * N + n0 + s) * H + i];
                        }
                        pr[K - 1] = ar[K - 1];
#pragma unroll
                        for (int j = K - 2; j >= 0; --j) {
                            ql[j] = fmaf(ar[j], ql[j + 1], g[j]);
                            pr[j] = ar[j] * pr[j + 1];
                        }
                        float P[1] = {pr[0]}, Q[1] = {ql[0]}, qin[1];
                        group_scan_left_any<LG>(P, Q, qin);
#pragma unroll
                        for (int j = 0; j < K; ++j) {
                            const float q = fmaf(pr[j], qin[0], ql[j]);
                            if constexpr (MP) {
                                if (j == 0 && p.qc_out != nullptr && l == 0 && act) p.qc_out[(map * N + n0 + s) * H + i] = a[0] * q;
                            }
                            float gc, du;                                  // gradient along the column recurrence, gradient of u
                            if constexpr (CF) {
                                gc = q + ga[s][j];
                                ga[s][j] = a[j] * gc;
                                du = gc;
                            } else {
                                gc = g[j];
                                du = q;
                            }
                            const float da = fmaf(gc, hprev[r][s][j], q * hhl[RECOMP ? 0 : r][s][j]);
                            const float t = da * a[j];
                            const float qB = du * Bv[j];
                            dAb[s] = fmaf(t, dl[j], dAb[s]);
                            if constexpr (LATEF) {
                                ddl[j] = fmaf(t, An[s], ddl[j]);
                                dxl[j] += qB;
                            } else {
                                ddl[j] = fmaf(t, An[s], fmaf(qB, xe[j], ddl[j]));
                                dxl[j] = fmaf(qB, dl[j], dxl[j]);
                            }
                            dBacc[r][s][j] = fmaf(du, dxe[j], dBacc[r][s][j]);
                        }
                    }
                    // sums over the states held by the other lane groups of this job
                    float* mine = part + (size_t)(step & 1) * 2 * THREADS * K + (size_t)slot * PANEL;
                    lds_write_k<LG, K>(mine, l, ddl);
                    lds_write_k<LG, K>(mine + THREADS * K, l, dxl);
                    __syncthreads();
                    if (act) {
                        const float* base = part + (size_t)(step & 1) * 2 * THREADS * K + (size_t)(slot - sg) * PANEL;
#pragma unroll
                        for (int v = 0; v < TT; ++v) {
                            if constexpr (!LATEF) {
                                const int t = tm + v * TMJ;
                                const int tens = t / PANEL, lc = t - tens * PANEL, col = cb + lc;
                                if (t < TASKS && col < W) {
                                    const float sum = sum_partials_fixed<PANEL, NG>(base + tens * (THREADS * K) + lds_colk<LG, K>(lc));
                                    if (tens == 0) {
                                        if constexpr (SP && !SPIN) ddw[ro + col] = sum;  // over the step of this cell, which nobody reads again
                                        else if constexpr (SPIN) {
                                            const float v = sum * dsoftplus_from_value(prow[lds_colk<LG, K>(lc)]);
                                            store_elem(ddm + ro + col, v);
                                            dBb += v;
                                        }
                                        else store_elem(ddm + ro + col, sum);
                                    } else {                                    // skip term; exactly +0 under the mask
                                        const float* cell = prow + lds_colk<LG, K>(lc);
                                        store_elem(dxm + ro + col, cell[4 * PANEL] != 0.0f ? 0.0f : fmaf(dsk, cell[3 * PANEL], sum));
                                    }
                                }
                                continue;
                            }
                            const int lc = tm + v * TMJ, col = cb + lc;
                            if (lc < PANEL && col < W) {
                                const int at = lds_colk<LG, K>(lc);
                                const float sA = sum_partials_fixed<PANEL, NG>(base + at);
                                const float sB = sum_partials_fixed<PANEL, NG>(base + THREADS * K + at);
                                const float* cell = prow + at;                  // dl, xe, dl*xe, dy, mask flag of this cell
                                const float dd = fmaf(cell[PANEL], sB, sA);
                                if constexpr (SP && !SPIN) ddw[ro + col] = dd;  // over the step of this cell, which nobody reads again
                                else if constexpr (SPIN) {
                                    const float v = dd * dsoftplus_from_value(cell[0]);
                                    store_elem(ddm + ro + col, v);
                                    dBb += v;
                                }
                                else store_elem(ddm + ro + col, dd);
                                // skip term; exactly +0 under the mask
                                store_elem(dxm + ro + col, cell[4 * PANEL] != 0.0f ? 0.0f : fmaf(dsk, cell[3 * PANEL], cell[0] * sB));
                            }
                        }
                    }
                    ++step;
                }
            }
#pragma unroll
            for (int s = 0; s < NW; ++s) {
#pragma unroll
                for (int j = 0; j < K; ++j) gaL[((size_t)ch * THREADS + tid) * (NW * K) + s * K + j] = ga[s][j];
                const float tot = group_sum_last<LG>(inside ? dAb[s] : 0.0f);
                if (l == LG - 1) dAL[((size_t)ch * SLOTS + slot) * NW + s] += tot;
            }
            {
                const float tot = group_sum_last<64>(dDb);
                if ((tid & 63) == 63) dDL[ch * WAVES + wave] += tot;
            }
            if constexpr (SPIN) {
                const float tot = group_sum_last<64>(dBb);
                if ((tid & 63) == 63) dBL[ch * WAVES + wave] += tot;
            }
        }

        // partial sums over this workgroup's channels, one write per band
        if (live) {
#pragma unroll
            for (int r = 0; r < RB; ++r) {
                const int i = r0 + r;
                if (i < H) {
#pragma unroll
                    for (int s = 0; s < NW; ++s) {
                        if (p.part_chunked) {                          // every lane stores; the reduction drops the columns past W
                            const size_t oc = ((((size_t)b * p.CG + cg) * N + n0 + s) * H + i) * PANEL + l * 4;
#pragma unroll
                            for (int j4 = 0; j4 < K / 4; ++j4) {
                                *reinterpret_cast<float4*>(p.pB + oc + j4 * (LG * 4)) =
                                    make_float4(dBacc[r][s][4 * j4], dBacc[r][s][4 * j4 + 1], dBacc[r][s][4 * j4 + 2], dBacc[r][s][4 * j4 + 3]);
                                *reinterpret_cast<float4*>(p.pC + oc + j4 * (LG * 4)) =
                                    make_float4(dCacc[r][s][4 * j4], dCacc[r][s][4 * j4 + 1], dCacc[r][s][4 * j4 + 2], dCacc[r][s][4 * j4 + 3]);
                            }
                            continue;
                        }
                        const size_t o = ((((size_t)b * p.CG + cg) * N + n0 + s) * H + i) * W;
                        if (nv == K) {
                            store_f32s<K>(p.pB + o + col0, dBacc[r][s]);
                            store_f32s<K>(p.pC + o + col0, dCacc[r][s]);
                        } else {
#pragma unroll
                            for (int j = 0; j < K; ++j)
                                if (col0 + j < W) { p.pB[o + col0 + j] = dBacc[r][s][j]; p.pC[o + col0 + j] = dCacc[r][s][j]; }
                        }
                    }
                }
            }
        }
    }

    // dA[b,c,n]: already summed over the lane group; dDskip[b,c]: the sum over the job's wavefronts, in index order
    __syncthreads();
    if (live && l == LG - 1) {
        for (int ch = 0; ch < nch; ++ch) {
#pragma unroll
            for (int s = 0; s < NW; ++s)
            {
                float* dst = p.pA + ((size_t)b * p.Dc + c_first + ch) * N + n0 + s;
                const float v = dAL[((size_t)ch * SLOTS + slot) * NW + s];
                *dst = (MP && p.accum) ? *dst + v : v;             // panels are launched one after the other
            }
        }
    }
    if (live && tm == 0 && p.pD != nullptr) {
        constexpr int WPJ = TMJ >= 64 ? TMJ / 64 : 1;     // wavefronts of a job
        const int w0 = (job_slot * TMJ) / 64;
        for (int ch = 0; ch < nch; ++ch) {
            float acc = 0.0f;
            for (int w = 0; w < WPJ; ++w) acc += dDL[ch * WAVES + w0 + w];
            float* dst = p.pD + (size_t)b * p.Dc + c_first + ch;
            *dst = (MP && p.accum) ? *dst + acc : acc;
        }
    }
    if constexpr (SPIN) {
        if (live && tm == 0 && p.pBias != nullptr) {
            constexpr int WPJ = TMJ >= 64 ? TMJ / 64 : 1;
            const int w0 = (job_slot * TMJ) / 64;
            for (int ch = 0; ch < nch; ++ch) {
                float acc = 0.0f;
                for (int w = 0; w < WPJ; ++w) acc += dBL[ch * WAVES + w0 + w];
                p.pBias[(size_t)b * p.Dc + c_first + ch] = acc;
            }
        }
    }
}

}  // namespace scan2d
