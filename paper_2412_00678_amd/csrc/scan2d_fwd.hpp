// Forward 2D selective scan kernel for gfx950 (2DMamba Eq. 3, Eq. 5, Eq. 6, y = C h + D x).
//
// Work decomposition (differs from the paper's sequential 2D tiles with carries in HBM):
//   * a "lane group" of LG lanes (LG = 16: one DPP row, LG = 64: a wavefront) owns a panel of
//     LG*K consecutive columns; lane l owns the K columns [l*K, l*K+K) and NW of the N states;
//   * the group walks down the rows.  The column recurrence (Eq. 6) is a plain FMA on
//     registers that persist from row to row, so the N-wide state never leaves VGPRs;
//   * the row recurrence (Eq. 5) is a serial chain over the lane's K columns plus one
//     log-step DPP scan of the per-lane (decay product, state) pairs across the group;
//   * a map uses NG = N / NW lane groups; their partial sums over states meet in LDS, one
//     barrier per row, and are summed in a fixed order;
//   * inputs of row i+1 are requested while row i is computed (a raw register is refilled
//     as soon as its content has been consumed).
// Maps wider than one panel are processed panel by panel, left to right; the row-end states
// of a panel travel to the next one through a small carry buffer (N floats per row).
#pragma once

#include <type_traits>

#include "scan2d_common.hpp"

namespace scan2d {

// Sum of the NG partial sums of one column (stride STRIDE floats), added in index order.  The
// loads are issued together for the common group counts so that their LDS latencies overlap.
template <int STRIDE, int G>
__device__ __forceinline__ float sum_partials_fixed(const float* p) {
    float v[G];
#pragma unroll
    for (int g = 0; g < G; ++g) v[g] = p[g * STRIDE];
    float acc = v[0];
#pragma unroll
    for (int g = 1; g < G; ++g) acc += v[g];
    return acc;
}
template <int STRIDE>
__device__ __forceinline__ float sum_partials(const float* p, int NG) {
    switch (NG) {
        case 2: return sum_partials_fixed<STRIDE, 2>(p);
        case 4: return sum_partials_fixed<STRIDE, 4>(p);
        case 8: return sum_partials_fixed<STRIDE, 8>(p);
        case 16: return sum_partials_fixed<STRIDE, 16>(p);
        default: {
            float acc = p[0];
            for (int g = 1; g < NG; ++g) acc += p[g * STRIDE];
            return acc;
        }
    }
}

struct FwdArgs {
    const void* x; const void* delta; const float* A; const void* Bm; const void* Cm;
    const float* Dskip; const uint8_t* mask; void* y;
    const float* delta_bias;   // [Dc] or null; read by the SP instantiations only (delta then holds the raw projection)
    const float* A_v = nullptr; // [Dc][N]; read by the AV instantiations only: decay parameter of the column recurrence
    float* carry;        // [maps][N][H] row-end states between column panels (panels > 1 only)
    float* ck = nullptr; // checkpoint sweep of the backward pass only: [maps][nb][N][W] column states entering each band
    const void* z = nullptr;     // GATE instantiations only: the block's gate branch, layout of x
    void* y_gated = nullptr;     // GATE instantiations only: y * SiLU(z); y itself may then be null (not stored)
    int nb = 0;          // bands of that sweep
    // checkpoint rows of LG*K floats in the lane order of the tiling, [K/4][LG][4]: every store instruction of a lane group
    // then writes 16 bytes x LG contiguously (the reader must have the same LG and K); 0: rows of W floats by column
    int ck_chunked = 0;
    long long maps;      // Bt * Dc
    int Dc, H, W, N;
    int NG;              // lane groups per map = ceil(N / NW)
    int MPW;             // maps per workgroup = (lane groups per workgroup) / NG, >= 1
    int panels;          // ceil(W / (LG * K))
    int RPB;             // rows between two workgroup barriers (1, 2, 4 or 8); sizes the dynamic LDS
};

// FAST (single-panel maps, any W): every lane reads its K columns with one wide buffer load per tensor.
// A lane that starts past the last column re-reads the columns of lane 0 and its results are
// discarded.  A lane that straddles the end of the row reads on into the next row (or zeros past the
// end of the tensor: the buffer descriptors carry the exact size): those cells sit to the right of
// every real column, so what they hold reaches no output (the row recurrence only runs rightwards,
// the column recurrence stays in its column), and they are never stored.  Buffer loads of dwords ignore
// the two low bits of the offset (measured: loads at other offsets return the dword below), so they need
// offsets that are multiples of 4 bytes: always so for fp32 rows, for bf16 rows of even width, and for mask
// rows when W is a multiple of 4 (MA).  The instantiations with MA = false request the aligned dwords around a
// lane's mask bytes and shift them into place (v_alignbyte_b32) where the row is unpacked - not where
// it is requested, which would wait for the load at once.  Without FAST (maps wider than one panel)
// every element access is guarded.
// UA (bf16 only): rows of odd width start on odd 2-byte boundaries every other row.  The loads fetch one
// dword more from the address rounded down to a dword and the K elements are shifted into place
// (v_alignbit_b32 by 0 or 16) where they are unpacked.
// MULTI: the map is wider than one panel (p.panels > 1); single-panel kernels carry no code
// for the panel hand-over.
// SP: the step is computed here, delta = softplus(raw + bias) (a second set of instantiations, so that
// the plain kernels carry neither the code nor its registers).
// WAVES: wavefronts per workgroup (4, 8 or 16).  A wave that is alone on its SIMD has nothing to cover
// its waits (loads, LDS, barriers, DPP chains) and these kernels then reach about half of the vector
// issue rate, so maps that are few but large spread their states over more waves (smaller NW) rather
// than leaving SIMDs with a single wave.
// VGPRs a kernel may spend on rows of loads in flight, per group of tensors.
#ifndef SCAN2D_PREFETCH_BUDGET_X
#define SCAN2D_PREFETCH_BUDGET_X 56
#endif
#ifndef SCAN2D_PREFETCH_BUDGET_S
#define SCAN2D_PREFETCH_BUDGET_S 48
#endif
constexpr int kPrefetchBudgetX = SCAN2D_PREFETCH_BUDGET_X, kPrefetchBudgetS = SCAN2D_PREFETCH_BUDGET_S;

// AV: the column recurrence (Eq. 6) uses a decay of its own, a_v = exp(step * A_v[c,n]) - the supplement's ablation
// of re-using A-bar for the vertical scan (one more exponential per state and column).
template <typename T, int LG, int K, int NW, int WAVES, bool EXACT, bool FAST, bool MULTI, bool SP = false, bool MA = true,
          bool UA = false, bool AV = false>
__global__ __launch_bounds__(WAVES * 64) void scan2d_fwd_kernel(const FwdArgs p) {
    static_assert(!UA || (FAST && !MA && Elem<T>::kBytes == 2), "UA: bf16 rows on odd 2-byte boundaries, unguarded loads");
    constexpr int SLOTS = WAVES * 64 / LG;
    constexpr int XW = words_of<T, K>();
    constexpr int PANEL = LG * K;
    constexpr int SC = (NW < 4 ? NW : (K >= 12 ? 2 : 4));   // states scanned together
    static_assert(NW % SC == 0, "state chunking");
    // partial sums over states: [2 buffers][RPB rows][SLOTS][PANEL]; the lane groups of a map
    // meet at a barrier once every RPB rows
    extern __shared__ float ypart[];
    const int RPB = p.RPB;

    const int tid = threadIdx.x;
    const int slot = tid / LG;
    const int l = tid % LG;
    const int NG = p.NG;
    int map_local = slot / NG;
    const int sg = slot - map_local * NG;
    const long long map0 = (long long)blockIdx.x * p.MPW;
    const bool live = (map_local < p.MPW) && (map0 + map_local < p.maps);
    if (!live) map_local = 0;                     // idle group: valid addresses, no writes
    const long long map = map0 + map_local;

    const int H = p.H, W = p.W, N = p.N;
    const size_t HW = (size_t)H * W;
    const int b0 = (int)(map0 / p.Dc);
    const int b = (int)(map / p.Dc), c = (int)(map % p.Dc);
    const int n0 = sg * NW;
    const int nvalid = EXACT ? NW : min(NW, N - n0);

    // Uniform bases (scalar registers) + 32-bit per-lane element offsets.
    const T* __restrict__ xu = reinterpret_cast<const T*>(p.x) + (size_t)map0 * HW;
    const T* __restrict__ du = reinterpret_cast<const T*>(p.delta) + (size_t)map0 * HW;
    T* __restrict__ yu = reinterpret_cast<T*>(p.y) + (size_t)map0 * HW;
    const T* __restrict__ Bu = reinterpret_cast<const T*>(p.Bm) + (size_t)b0 * N * HW;
    const T* __restrict__ Cu = reinterpret_cast<const T*>(p.Cm) + (size_t)b0 * N * HW;
    const uint8_t* __restrict__ mu = p.mask ? p.mask + (size_t)b0 * HW : nullptr;
    const uint32_t xlane = (uint32_t)(map_local * HW);
    const uint32_t slane = (uint32_t)(((size_t)(b - b0) * N + n0) * HW);
    const uint32_t mlane = (uint32_t)((size_t)(b - b0) * HW);
    constexpr size_t EBY = (size_t)Elem<T>::kBytes;
    const size_t left_maps = (size_t)(p.maps - map0) * HW, left_items = (size_t)(p.maps / p.Dc - b0) * HW;
    // Exact sizes, rounded up to whole dwords: a load whose dword is only partly inside the range would
    // return 0 for all of it, and the last dword of a tensor with an odd number of bf16 elements, or of a
    // mask whose size is not a multiple of 4, holds real data (the dword itself lies in mapped memory:
    // its first bytes are the tensor's).
    auto up4 = [](size_t bytes) { return (bytes + 3) & ~(size_t)3; };
    const rsrc_t rsx = make_rsrc(xu, up4(left_maps * EBY)), rsd = make_rsrc(du, up4(left_maps * EBY)),
                 rsB = make_rsrc(Bu, up4(left_items * N * EBY)), rsC = make_rsrc(Cu, up4(left_items * N * EBY)),
                 rsm = make_rsrc(mu, up4(left_items));

    float Ap[NW], Avp[NW];
#pragma unroll
    for (int s = 0; s < NW; ++s) {
        const int n = (EXACT || s < nvalid) ? n0 + s : n0;
        Ap[s] = p.A[(size_t)c * N + n] * kLog2e;             // a = exp2(delta * A * log2 e)
        Avp[s] = AV ? p.A_v[(size_t)c * N + n] * kLog2e : 0.0f;
    }
    const float dsk = (p.Dskip != nullptr && sg == 0) ? p.Dskip[c] : 0.0f;
    // SP: `delta` holds the raw projection and the step is softplus(raw + delta_bias[c]) (Eq. 3)
    const float dbias = (SP && p.delta_bias != nullptr) ? p.delta_bias[c] : 0.0f;
    const bool reduce = NG > 1;

    int step = 0;   // rows processed so far: its parity selects the LDS buffer
    const int panels = MULTI ? p.panels : 1;
    for (int panel = 0; panel < panels; ++panel) {
        if (panel > 0) __threadfence();           // row-end states of the previous panel are visible
        const int col0 = panel * PANEL + l * K;
        const bool inside = col0 < W;
        const uint32_t lcol = (FAST && !inside) ? 0u : (uint32_t)col0;   // FAST: idle lanes mirror lane 0

        float h[NW][K];
#pragma unroll
        for (int s = 0; s < NW; ++s)
#pragma unroll
            for (int j = 0; j < K; ++j) h[s][j] = 0.0f;       // h[-1, j] = 0

        // Raw registers of the rows in flight.  The row loop below is written for TRIP rows per
        // trip; PDX (x, delta, mask: one stream per channel, straight from HBM) and PDS (Bm, Cm: shared
        // by the channels, mostly L2 hits) say how many rows ahead each group of loads runs.  Every
        // row of depth costs another set of raw registers, so the depth follows the size of a set.
        constexpr int XSET = 2 * XW + K / 4, SSET = 2 * NW * XW;
        constexpr int PDX = 4 * XSET <= kPrefetchBudgetX ? 4 : (2 * XSET <= kPrefetchBudgetX ? 2 : 1);
        constexpr int PDS = 4 * SSET <= kPrefetchBudgetS ? 4 : (2 * SSET <= kPrefetchBudgetS ? 2 : 1);
        constexpr int TRIP = PDX > PDS ? PDX : PDS;
        constexpr int XWR = XW + (UA ? 1 : 0);                 // raw dwords per lane and tensor row
        constexpr int MWR = K / 4 + ((FAST && !MA) ? 1 : 0);   // raw mask dwords: one more when the bytes are shifted into place
        uint32_t rx[PDX][XWR], rd[PDX][XWR], rm[PDX][MWR], rB[PDS][NW][XWR], rC[PDS][NW][XWR];
        // FAST: buffer addressing - uniform base and uniform row offset in scalar registers, one
        // loop-invariant 32-bit byte offset per lane (the host bounds the span to 2^31 bytes)
        constexpr uint32_t EB = (uint32_t)Elem<T>::kBytes;
        auto ld = [&](const T* base, rsrc_t rs, uint32_t uni_off, uint32_t lane_off, uint32_t* r) {
            if constexpr (FAST && UA) buffer_load_words<XWR>(rs, ((lane_off + lcol + uni_off) * EB) & ~3u, 0u, r);   // rounded down to a dword
            else if constexpr (FAST) buffer_load_words<XW>(rs, (lane_off + lcol) * EB, uni_off * EB, r);
            else load_row<T, K>(base + uni_off + lane_off, col0, W, false, r);
        };
        auto ldm = [&](uint32_t uni_off, uint32_t* r) {
            if constexpr (FAST) {
                if constexpr (MA) buffer_load_words<K / 4>(rsm, mlane + lcol, uni_off, r);
                else buffer_load_words<MWR>(rsm, (mlane + lcol + uni_off) & ~3u, 0u, r);   // the aligned dwords around the K bytes
            }
            else load_mask<K>(mu + uni_off + mlane, col0, W, false, r);
        };
        // State s of this lane group: uniform offset s*HW when every group is full; otherwise a
        // per-lane offset, with the idle states of a ragged last group re-reading state n0.
        auto lds = [&](const T* base, rsrc_t rs, int s, uint32_t row_off, uint32_t* r) {
            if constexpr (EXACT) ld(base, rs, (uint32_t)s * (uint32_t)HW + row_off, slane, r);
            else ld(base, rs, row_off, slane + (uint32_t)((s < nvalid ? s : 0) * HW), r);
        };
        // UA: the K elements of a raw register set, shifted into place; the element offset of the load
        // (uniform + lane part) says whether it started on an odd 2-byte boundary
        auto unpack = [&](const uint32_t* raw, uint32_t uni_off, uint32_t lane_off, uint32_t* out) {
            if constexpr (UA) {
                const uint32_t sh = ((uni_off ^ (lane_off + lcol)) & 1u) << 4;
#pragma unroll
                for (int w = 0; w < XW; ++w) out[w] = __builtin_amdgcn_alignbit(raw[w + 1], raw[w], sh);
            } else {
#pragma unroll
                for (int w = 0; w < XW; ++w) out[w] = raw[w];
            }
        };
        auto unpacks = [&](const uint32_t* raw, int s, uint32_t row_off, uint32_t* out) {
            if constexpr (EXACT) unpack(raw, (uint32_t)s * (uint32_t)HW + row_off, slane, out);
            else unpack(raw, row_off, slane + (uint32_t)((s < nvalid ? s : 0) * HW), out);
        };
#pragma unroll
        for (int d = 0; d < PDX; ++d) {
            const uint32_t ro = (uint32_t)min(d, H - 1) * (uint32_t)W;
            ld(xu, rsx, ro, xlane, rx[d]);
            ld(du, rsd, ro, xlane, rd[d]);
#pragma unroll
            for (int w = 0; w < MWR; ++w) rm[d][w] = 0u;
            if (mu) ldm(ro, rm[d]);
        }
#pragma unroll
        for (int d = 0; d < PDS; ++d) {
            const uint32_t ro = (uint32_t)min(d, H - 1) * (uint32_t)W;
#pragma unroll
            for (int s = 0; s < NW; ++s) {
                lds(Bu, rsB, s, ro, rB[d][s]);
                lds(Cu, rsC, s, ro, rC[d][s]);
            }
        }

        // One row; PAR = position of the row inside the trip (selects the raw register sets).
        auto do_row = [&](const int i, auto par) __attribute__((always_inline)) {
            constexpr int PAR = decltype(par)::value;
            constexpr int XS = PAR % PDX, SS = PAR % PDS;
            // a row past the end re-reads the last row
            const uint32_t nxt_x = (uint32_t)min(i + PDX, H - 1) * (uint32_t)W;
            const uint32_t nxt_s = (uint32_t)min(i + PDS, H - 1) * (uint32_t)W;
            float dl[K], dx[K], yacc[K];
            const uint32_t cur = (uint32_t)i * (uint32_t)W;
            uint32_t ux[XW], ud[XW], um[K / 4];
            unpack(rx[XS], cur, xlane, ux);
            unpack(rd[XS], cur, xlane, ud);
            if constexpr (FAST && !MA) {              // the K mask bytes, shifted into place where they are used, not where they are requested
                const uint32_t sh = (mlane + lcol + cur) & 3u;
#pragma unroll
                for (int w = 0; w < K / 4; ++w) um[w] = __builtin_amdgcn_alignbyte(rm[XS][w + 1], rm[XS][w], sh);
            } else {
#pragma unroll
                for (int w = 0; w < K / 4; ++w) um[w] = rm[XS][w];
            }
#pragma unroll
            for (int j = 0; j < K; ++j) {
                dl[j] = get_elem<T, K>(ud, j);
                if constexpr (SP) dl[j] = softplus_f32(dl[j] + dbias);
                const float xv = get_elem<T, K>(ux, j);
                const float xe = mask_bit<K>(um, j) ? 0.0f : xv;          // select: nothing under the mask leaks
                dx[j] = dl[j] * xe;
                yacc[j] = dsk * xe;
            }
            ld(xu, rsx, nxt_x, xlane, rx[XS]);
            ld(du, rsd, nxt_x, xlane, rd[XS]);
            if (mu) ldm(nxt_x, rm[XS]);

#pragma unroll
            for (int s0 = 0; s0 < NW; s0 += SC) {
                if (EXACT || s0 < nvalid) {       // a ragged last group idles whole chunks only when SC divides
                    float a[SC][K], hl[SC][K], pl[SC][K];
                    float P[SC], Hh[SC], cin[SC];
#pragma unroll
                    for (int t = 0; t < SC; ++t) {
                        const int s = s0 + t;
#pragma unroll
                        for (int j = 0; j < K; ++j) a[t][j] = __builtin_amdgcn_exp2f(dl[j] * Ap[s]);
                        uint32_t uB[XW];
                        unpacks(rB[SS][s], s, cur, uB);
                        hl[t][0] = dx[0] * get_elem<T, K>(uB, 0);
                        pl[t][0] = a[t][0];
                        if (MULTI && panel > 0 && l == 0) {   // state entering from the panel to the left
                            const float* cw = p.carry + ((size_t)map * N + n0 + ((EXACT || s < nvalid) ? s : 0)) * H + i;
                            hl[t][0] = fmaf(a[t][0], __hip_atomic_load(cw, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT), hl[t][0]);
                        }
#pragma unroll
                        for (int j = 1; j < K; ++j) {
                            hl[t][j] = fmaf(a[t][j], hl[t][j - 1], dx[j] * get_elem<T, K>(uB, j));
                            pl[t][j] = pl[t][j - 1] * a[t][j];
                        }
                        lds(Bu, rsB, s, nxt_s, rB[SS][s]);
                        P[t] = pl[t][K - 1];
                        Hh[t] = hl[t][K - 1];
                    }
                    group_scan<LG, SC>(P, Hh, cin);
#pragma unroll
                    for (int t = 0; t < SC; ++t) {
                        const int s = s0 + t;
                        if (MULTI && panel + 1 < p.panels && l == LG - 1 && live && (EXACT || s < nvalid)) {
                            float* cw = p.carry + ((size_t)map * N + n0 + s) * H + i;
                            __hip_atomic_store(cw, Hh[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        }
                        const float cmul = (EXACT || s < nvalid) ? 1.0f : 0.0f;   // idle state adds nothing to y
                        uint32_t uC[XW];
                        unpacks(rC[SS][s], s, cur, uC);
#pragma unroll
                        for (int j = 0; j < K; ++j) {
                            // Eq. 5; at the lane's last column the scan result is the state itself
                            const float hh = (j == K - 1) ? Hh[t] : fmaf(pl[t][j], cin[t], hl[t][j]);
                            // Eq. 6.  AV: plain fmaf - the one-line asm hides its operands from the compiler's hazard
                            // handling, and a transcendental result may not be read by the very next instruction
                            if constexpr (AV) h[s][j] = fmaf(__builtin_amdgcn_exp2f(dl[j] * Avp[s]), h[s][j], hh);
                            else fma_inplace(h[s][j], a[t][j], hh);
                            const float cv = EXACT ? get_elem<T, K>(uC, j) : cmul * get_elem<T, K>(uC, j);
                            yacc[j] = fmaf(cv, h[s][j], yacc[j]);
                        }
                        lds(Cu, rsC, s, nxt_s, rC[SS][s]);
                    }
                }
            }

            T* yrow = yu + (size_t)i * W;
            if (!reduce) {
                if (live) {
                    if constexpr (FAST) {
                        if (inside) store_row<T, K>(yrow + xlane, col0, W, !UA, yacc);   // wide unless it straddles the row end
                    } else {
                        store_row<T, K>(yrow + xlane, col0, W, false, yacc);
                    }
                }
            } else {
                const int batch = step / RPB, rb = step - batch * RPB;     // row inside the current batch
                float* buf = ypart + (size_t)(batch & 1) * RPB * SLOTS * PANEL;
                float* mine = buf + ((size_t)rb * SLOTS + slot) * PANEL + l * K;
#pragma unroll
                for (int j = 0; j < K; ++j) mine[j] = yacc[j];
                if (rb == RPB - 1 || i == H - 1) {                         // uniform: batch complete
                    __syncthreads();
                    if (live) {
                        // the (row, column) outputs of the batch are dealt out over all threads of the map, not row by
                        // row: with fewer columns than threads a row would keep only the first lane groups busy
                        const float* base0 = buf + (size_t)(slot - sg) * PANEL;       // first group of this map, first row
                        for (int idx = sg * LG + l; idx < (rb + 1) * PANEL; idx += NG * LG) {
                            const int r = idx / PANEL, col = idx - r * PANEL;
                            const int gc = panel * PANEL + col;
                            if (gc < W)
                                store_elem(yrow - (size_t)(rb - r) * W + xlane + gc,
                                           sum_partials<PANEL>(base0 + (size_t)r * SLOTS * PANEL + col, NG));
                        }
                    }
                    step += RPB - 1 - rb;                                  // a short last batch still ends its buffer
                }
            }
            ++step;
        };
        // Full trips run without a test between their rows: every path through the loop body then
        // issues the same loads, and the compiler's wait counts let all TRIP rows of loads stay in
        // flight (a skippable row would make it wait for nearly everything at each row).
        int i = 0;
        for (; i + TRIP <= H; i += TRIP) {
            do_row(i, std::integral_constant<int, 0>{});
            if constexpr (TRIP >= 2) do_row(i + 1, std::integral_constant<int, 1>{});
            if constexpr (TRIP >= 4) {
                do_row(i + 2, std::integral_constant<int, 2>{});
                do_row(i + 3, std::integral_constant<int, 3>{});
            }
        }
        if (i < H) {                                          // the last H % TRIP rows
            do_row(i, std::integral_constant<int, 0>{});
            if constexpr (TRIP >= 2) { if (i + 1 < H) do_row(i + 1, std::integral_constant<int, 1>{}); }
            if constexpr (TRIP >= 4) { if (i + 2 < H) do_row(i + 2, std::integral_constant<int, 2>{}); }
        }
    }
}

}  // namespace scan2d
