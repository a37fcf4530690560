// Backward 2D selective scan kernels for gfx950 (2DMamba Supp. B: two forward scans rebuild the
// states, a reverse column scan and a reverse row scan carry the gradients).
//
// The forward pass stores nothing N-wide, so the backward works in bands of RB rows:
//   1. a checkpoint kernel repeats the forward recurrences and keeps only the column state h
//      at the top of every band (N*W floats per band and map);
//   2. the main kernel walks the bands from the bottom up.  Per band and channel it rebuilds
//      h[i-1,j] and hhor[i,j-1] for the band's rows into registers (scans 1 and 2), then walks
//      the band's rows upwards with the reverse column recurrence g (a plain FMA on a register
//      that persists from row to row) and the reverse row recurrence q (serial over the lane's
//      K columns plus a leftward lane-group scan), and forms the local gradients;
//   3. sums over channels (dBm, dCm) are accumulated in registers over the GS channels a
//      workgroup handles one after the other, written once per band as partial sums, and added
//      up over the channel groups by a reduction kernel in a fixed order; dA and dDskip are
//      reduced over lanes in a fixed order and over batch items by the same kernel.
// Lane mapping is that of the forward kernel: a lane group of LG lanes owns LG*K columns, lane l
// the columns [l*K, l*K+K) and NW states; NG = ceil(N/NW) lane groups share a map and meet in
// LDS once per row for the sums over states (ddelta, dx).
// All accesses are unguarded and wide.  A lane past the last column mirrors lane 0 with dy
// forced to 0, so nothing flows out of it into the reverse scans, and it never stores.
// FAST = W is a multiple of K.  Without it the lane that holds the last column reads on into
// the next row; its cells past the row end get dy = 0 and a zero column state, which makes every
// gradient they could contribute exactly 0 whatever finite values they hold, and it stores
// element by element.  The one row behind which a tensor ends (the last row of its last map) is
// read from a padded copy that a small kernel leaves in the workspace (`tail`): the row pointer is
// a select, so that no load sits in a branch (loads in branches make the compiler's wait counts
// conservative, which cost these instantiations a quarter of their speed).
// SP: the caller's step is softplus(raw + delta_bias[c]) (Eq. 3).  A kernel of its own has written it
// once per position as fp32 (`delta` points there, whatever the storage type T), because each of a map's
// lane groups would otherwise repeat the softplus in both sweeps.  The main sweep writes the gradient of
// the step, unrounded, over the step itself (a row's step is not read again once its gradient is stored),
// and a last element-wise kernel applies the chain rule there - inside the sweep it would put a dependent
// global load behind every row's barrier (a second set of instantiations).
// PF: the inputs of the next row are requested before the current row is processed (costs one
// more row of raw registers); without it the kernel relies on several waves per SIMD.
#pragma once

#include "scan2d_common.hpp"
#include "scan2d_fwd.hpp"   // sum_partials

namespace scan2d {

struct BwdArgs {
    const void* x; const void* delta; const float* A; const void* Bm; const void* Cm;
    const float* Dskip; const uint8_t* mask; const void* dy;
    const float* delta_bias;   // [Dc] or null; read by the single-panel shared-producer sweeps (SP), which apply the softplus themselves
    void* dx; void* ddelta;
    float* ck;           // [maps][nb][N][W]   column state entering each band (band 0 unused)
    int ck_chunked = 0;  // shared-producer sweeps only: rows of LG*K floats in lane order [K/4][LG][4] (see FwdArgs)
    int part_chunked = 0; // shared-producer main sweep, CG > 1: the rows of pB / pC in the same lane order (the reduction
                         // kernel puts the columns back in place)
    float* pB; float* pC; // [Bt][CG][N][H][W] partial sums over the channels of one group
    const void* tail;    // padded copies of the rows behind which the tensors end (instantiations without FAST)
    float* pA;           // [Bt][Dc][N]
    float* pD;           // [Bt][Dc]
    // GATE instantiations of the shared-producer sweep only: the block's output gate inside the sweep
    const void* z = nullptr;        // gate branch, layout of x
    const void* y_scan = nullptr;   // the stored scan output, layout of x
    void* dz = nullptr;             // gradient of z, layout of x
    float* pBias = nullptr; // [Bt][Dc] sums of ddelta_raw per map, written by the sweeps that apply the softplus themselves (or null)
    int Bt, Dc, H, W, N;
    int NG;              // lane groups per map
    int GS;              // channels a workgroup handles one after the other
    int CG;              // channel groups = ceil(Dc / GS)
    int nb;              // bands = ceil(H / RB)
    // Maps wider than one lane-group panel are swept panel by panel (one launch each).  The row recurrences cross
    // the panel borders through carry buffers [maps][N][H]: the checkpoint sweeps run left to right and hand on the
    // row-end states hhor, the main sweeps run right to left and hand on a*q of their first column.
    int cb = 0;                          // first column of this launch's panel
    const float* hc_in = nullptr;        // row-end states of the panel to the left (null: first panel)
    float* hc_out = nullptr;             // checkpoint sweep: row-end states of this panel (null: last panel)
    const float* qc_in = nullptr;        // main sweep: a*q entering from the panel to the right (null: last panel)
    float* qc_out = nullptr;             // main sweep: a*q of this panel's first column (null: first panel)
    int accum = 0;                       // main sweep: add to pA / pD instead of overwriting them (all but the first launch)
    // AV instantiations only (independent decay of the column recurrence, the supplement's A-bar ablation)
    const float* A_v = nullptr;          // [Dc][N]
    float* pAv = nullptr;                // [Bt][Dc][N] partial sums of dA_v
};

template <int K>
__device__ __forceinline__ void load_f32s(const float* __restrict__ p, float* v) {
    uint32_t r[K];
    load_words<K>(reinterpret_cast<const uint32_t*>(p), r);
#pragma unroll
    for (int j = 0; j < K; ++j) v[j] = __uint_as_float(r[j]);
}
template <int K>
__device__ __forceinline__ void store_f32s(float* __restrict__ p, const float* v) {
    uint32_t r[K];
#pragma unroll
    for (int j = 0; j < K; ++j) r[j] = __float_as_uint(v[j]);
    store_words<K>(reinterpret_cast<uint32_t*>(p), r);
}

// K elements of one row for this lane (see FAST above), read wide from any byte address.  Without
// FAST the lane that holds the last column reads past the row end; `last` says that this is the row
// behind which the tensor ends, and the padded copy `tail_row` is read instead.
template <typename T, int K, bool FAST>
__device__ __forceinline__ void ld_elems(const T* rowp, uint32_t lcol, bool last, const T* tail_row, uint32_t* r) {
    const T* q = rowp;
    if constexpr (!FAST) q = last ? tail_row : rowp;
    load_words_any<words_of<T, K>()>(q + lcol, r);
}
template <int K, bool FAST>
__device__ __forceinline__ void ld_mask(const uint8_t* rowp, uint32_t lcol, bool last, const uint8_t* tail_row, uint32_t* r) {
    if (rowp == nullptr) {
#pragma unroll
        for (int w = 0; w < K / 4; ++w) r[w] = 0u;
    } else {
        const uint8_t* q = rowp;
        if constexpr (!FAST) q = last ? tail_row : rowp;
        load_words_any<K / 4>(q + lcol, r);
    }
}
// Layout of the padded copies: five rows of W + 16 elements (x, delta, dy, Bm, Cm) and one of W + 16
// mask bytes; each holds the last row of the last map / state plane of its tensor, zeros behind it.
template <typename T>
struct TailRows {
    const T *x, *delta, *dy, *B, *C;
    const uint8_t* mask;
    __device__ __forceinline__ TailRows(const void* base, int W) {
        const T* t = static_cast<const T*>(base);
        const size_t ts = (size_t)W + 16;
        x = t; delta = t + ts; dy = t + 2 * ts; B = t + 3 * ts; C = t + 4 * ts;
        mask = reinterpret_cast<const uint8_t*>(t + 5 * ts);
    }
};

// ---------------------------------------------------------------------------- checkpoint sweep
// CF (columns first, single panel only): the state that persists from row to row is v = a * v[i-1,j] + u, which
// needs no row scan at all.
template <typename T, int LG, int K, int NW, int WAVES, int RB, bool FAST, bool SP = false, bool AV = false, bool CF = false>
__global__ __launch_bounds__(WAVES * 64) void scan2d_bwd_ckpt_kernel(const BwdArgs p) {
    static_assert(!(CF && AV), "columns first has one decay");
    constexpr int SLOTS = WAVES * 64 / LG;
    constexpr int XW = words_of<T, K>();
    using DT = std::conditional_t<SP, float, T>;              // element type of the step
    constexpr int XWD = words_of<DT, K>();
    const int tid = threadIdx.x, slot = tid / LG, l = tid % LG;
    const int NG = p.NG, MPW = SLOTS / NG;
    const int map_local = slot / NG, sg = slot - map_local * NG;
    const long long maps = (long long)p.Bt * p.Dc;
    const long long map = (long long)blockIdx.x * MPW + map_local;
    if (map_local >= MPW || map >= maps) return;             // no barriers in this kernel
    const int H = p.H, W = p.W, N = p.N;
    const size_t HW = (size_t)H * W;
    const int b = (int)(map / p.Dc), c = (int)(map % p.Dc);
    const int n0 = sg * NW, nvalid = min(NW, N - n0);
    const int col0 = p.cb + l * K;
    const bool inside = col0 < W;
    const uint32_t lcol = inside ? (uint32_t)col0 : (uint32_t)p.cb;
    const T* xm = reinterpret_cast<const T*>(p.x) + (size_t)map * HW;
    const DT* dm = reinterpret_cast<const DT*>(p.delta) + (size_t)map * HW;
    const uint8_t* mm = p.mask ? p.mask + (size_t)b * HW : nullptr;
    const T* Bs[NW];
    float Ap[NW], Avp[NW], h[NW][K];
#pragma unroll
    for (int s = 0; s < NW; ++s) {
        const int n = n0 + (s < nvalid ? s : 0);
        Bs[s] = reinterpret_cast<const T*>(p.Bm) + ((size_t)b * N + n) * HW;
        Ap[s] = p.A[(size_t)c * N + n] * kLog2e;
        Avp[s] = AV ? p.A_v[(size_t)c * N + n] * kLog2e : 0.0f;
#pragma unroll
        for (int j = 0; j < K; ++j) h[s][j] = 0.0f;
    }
    // x, delta, mask (one HBM stream per channel) run PDX rows ahead in a ring of raw registers, Bm one
    // row ahead; the row loop is written as trips of PDX rows without a test between them, so that
    // the wait counts the compiler derives let all of them stay in flight.
    constexpr int PDX = (XW + XWD + K / 4 <= 28) ? 2 : 1;
    constexpr int SC = NW >= 4 ? 4 : NW;                      // states scanned together
    uint32_t rx[PDX][XW], rd[PDX][XWD], rm[PDX][K / 4], rB[NW][XW];
    const int last = p.hc_out != nullptr ? H - 1 : H - 2;     // the last row's state is never needed, its row-end state is
    // without FAST: is this lane's map / state plane / batch item the last of its tensor?  (the step of
    // the SP instantiations lives in the workspace, which has room behind it)
    const TailRows<T> tl(p.tail, W);
    const bool lastx = map == maps - 1, lastm = b == p.Bt - 1;
    bool lastB[NW];
#pragma unroll
    for (int s = 0; s < NW; ++s) lastB[s] = lastm && (n0 + (s < nvalid ? s : 0) == N - 1);
#pragma unroll
    for (int d = 0; d < PDX; ++d) {
        const int row = min(d, H - 1);
        const size_t ro = (size_t)row * W;
        ld_elems<T, K, FAST>(xm + ro, lcol, lastx && row == H - 1, tl.x, rx[d]);
        ld_elems<DT, K, FAST>(dm + ro, lcol, !SP && lastx && row == H - 1, reinterpret_cast<const DT*>(tl.delta), rd[d]);
        ld_mask<K, FAST>(mm ? mm + ro : nullptr, lcol, lastm && row == H - 1, tl.mask, rm[d]);
    }
#pragma unroll
    for (int s = 0; s < NW; ++s) ld_elems<T, K, FAST>(Bs[s], lcol, lastB[s] && H == 1, tl.B, rB[s]);

    auto do_row = [&](const int i, auto par) __attribute__((always_inline)) {
        constexpr int XS = decltype(par)::value % PDX;
        const int row_x = min(i + PDX, H - 1), row_s = min(i + 1, H - 1);   // a row past the end re-reads the last row
        const size_t nxt_x = (size_t)row_x * W;
        const size_t nxt_s = (size_t)row_s * W;
        float dl[K], dxe[K];
#pragma unroll
        for (int j = 0; j < K; ++j) {
            dl[j] = get_elem<DT, K>(rd[XS], j);
            const float xe = mask_bit<K>(rm[XS], j) ? 0.0f : get_elem<T, K>(rx[XS], j);
            dxe[j] = dl[j] * xe;
        }
        ld_elems<T, K, FAST>(xm + nxt_x, lcol, lastx && row_x == H - 1, tl.x, rx[XS]);
        ld_elems<DT, K, FAST>(dm + nxt_x, lcol, !SP && lastx && row_x == H - 1, reinterpret_cast<const DT*>(tl.delta), rd[XS]);
        ld_mask<K, FAST>(mm ? mm + nxt_x : nullptr, lcol, lastm && row_x == H - 1, tl.mask, rm[XS]);
        if constexpr (CF) {
#pragma unroll
            for (int s = 0; s < NW; ++s) {
#pragma unroll
                for (int j = 0; j < K; ++j)
                    h[s][j] = fmaf(__builtin_amdgcn_exp2f(dl[j] * Ap[s]), h[s][j], dxe[j] * get_elem<T, K>(rB[s], j));
                ld_elems<T, K, FAST>(Bs[s] + nxt_s, lcol, lastB[s] && row_s == H - 1, tl.B, rB[s]);
            }
        }
#pragma unroll
        for (int s0 = 0; s0 < (CF ? 0 : NW); s0 += SC) {
            float a[SC][K], hl[SC][K], pl[SC][K], P[SC], Hh[SC], cin[SC];
#pragma unroll
            for (int t = 0; t < SC; ++t) {
                const int s = s0 + t;
#pragma unroll
                for (int j = 0; j < K; ++j) a[t][j] = __builtin_amdgcn_exp2f(dl[j] * Ap[s]);
                hl[t][0] = dxe[0] * get_elem<T, K>(rB[s], 0);
                pl[t][0] = a[t][0];
                if (p.hc_in != nullptr && l == 0)             // state entering from the panel to the left
                    hl[t][0] = fmaf(a[t][0], p.hc_in[((size_t)map * N + n0 + (s < nvalid ? s : 0)) * H + i], hl[t][0]);
#pragma unroll
                for (int j = 1; j < K; ++j) {
                    hl[t][j] = fmaf(a[t][j], hl[t][j - 1], dxe[j] * get_elem<T, K>(rB[s], j));
                    pl[t][j] = pl[t][j - 1] * a[t][j];
                }
                ld_elems<T, K, FAST>(Bs[s] + nxt_s, lcol, lastB[s] && row_s == H - 1, tl.B, rB[s]);
                P[t] = pl[t][K - 1];
                Hh[t] = hl[t][K - 1];
            }
            group_scan<LG, SC>(P, Hh, cin);
            if (p.hc_out != nullptr && l == LG - 1) {         // row-end states of this panel (a panel with a successor is full)
#pragma unroll
                for (int t = 0; t < SC; ++t)
                    if (s0 + t < nvalid) p.hc_out[((size_t)map * N + n0 + s0 + t) * H + i] = Hh[t];
            }
#pragma unroll
            for (int t = 0; t < SC; ++t) {
#pragma unroll
                for (int j = 0; j < K; ++j) {
                    const float hh = (j == K - 1) ? Hh[t] : fmaf(pl[t][j], cin[t], hl[t][j]);
                    if constexpr (AV) h[s0 + t][j] = fmaf(__builtin_amdgcn_exp2f(dl[j] * Avp[s0 + t]), h[s0 + t][j], hh);   // no asm behind a transcendental
                    else fma_inplace(h[s0 + t][j], a[t][j], hh);
                }
            }
        }
        if ((i + 1) % RB == 0 && i + 1 < H) {                 // h[i] enters band (i+1)/RB
            const int band = (i + 1) / RB;
#pragma unroll
            for (int s = 0; s < NW; ++s) {
                if (s < nvalid) {
                    float* dst = p.ck + (((size_t)map * p.nb + band) * N + n0 + s) * W;
                    if (FAST ? inside : col0 + K <= W) {
                        store_f32s<K>(dst + col0, h[s]);
                    } else if (!FAST) {
#pragma unroll
                        for (int j = 0; j < K; ++j)
                            if (col0 + j < W) dst[col0 + j] = h[s][j];
                    }
                }
            }
        }
    };
    int i = 0;
    for (; i + PDX - 1 <= last; i += PDX) {
        do_row(i, std::integral_constant<int, 0>{});
        if constexpr (PDX == 2) do_row(i + 1, std::integral_constant<int, 1>{});
    }
    if constexpr (PDX == 2) { if (i <= last) do_row(i, std::integral_constant<int, 0>{}); }
}

// ---------------------------------------------------------------------------------- main sweep
// Dynamic LDS layout (floats), T = workgroup threads:
//   part [2][2][T*K]   per-thread partial sums over its states of ddelta and dx (double buffered)
//   gaL  [GS][T*NW*K]  a[i+1,j]*g[i+1,j] of every channel, kept between bands
//   dAL  [GS][T*NW]    per-lane partial of dA
//   dDL  [GS][T]       per-lane partial of dDskip (first lane group of a map only)
// AV: the column recurrence has its own decay a_v = exp(step * A_v[c,n]); the gradient through the decays splits
// into the row part q * hhor[i,j-1] (to A) and the column part g * h[i-1,j] (to A_v).
template <typename T, int LG, int K, int NW, int WAVES, int RB, bool FAST, bool PF, bool SP = false, bool AV = false>
__global__ __launch_bounds__(WAVES * 64) void scan2d_bwd_main_kernel(const BwdArgs p) {
    constexpr int THREADS = WAVES * 64;
    constexpr int SLOTS = THREADS / LG;
    constexpr int XW = words_of<T, K>();
    using DT = std::conditional_t<SP, float, T>;         // element type of the step
    constexpr int XWD = words_of<DT, K>();
    constexpr int PANEL = LG * K;
    extern __shared__ float lds[];
    const int GS = p.GS;
    float* part = lds;                                   // [2][2][SLOTS][PANEL]
    float* gaL = part + 4 * THREADS * K;                 // [GS][THREADS][NW*K]
    float* dAL = gaL + (size_t)GS * THREADS * NW * K;    // [GS][THREADS][NW]
    float* dDL = dAL + (size_t)GS * THREADS * NW;        // [GS][THREADS]
    float dVtot[NW];                                     // AV (one channel per workgroup): per-lane partial of dA_v over all bands
#pragma unroll
    for (int s = 0; s < NW; ++s) dVtot[s] = 0.0f;

    const int tid = threadIdx.x, slot = tid / LG, l = tid % LG;
    const int NG = p.NG, JPW = SLOTS / NG;               // jobs (batch item, channel group) per workgroup
    int job_local = slot / NG;
    const int sg = slot - job_local * NG;
    const long long jobs = (long long)p.Bt * p.CG;
    const long long job0 = (long long)blockIdx.x * JPW;
    const bool live = (job_local < JPW) && (job0 + job_local < jobs);
    if (!live) job_local = 0;
    const long long job = job0 + job_local;
    const int b = (int)(job / p.CG), cg = (int)(job % p.CG);
    const int c_first = cg * GS;
    const int nch = live ? min(GS, p.Dc - c_first) : 0;

    const int H = p.H, W = p.W, N = p.N;
    const size_t HW = (size_t)H * W;
    const int n0 = sg * NW, nvalid = min(NW, N - n0);
    const int col0 = p.cb + l * K;
    const bool inside = col0 < W;
    const uint32_t lcol = inside ? (uint32_t)col0 : (uint32_t)p.cb;
    const TailRows<T> tl(p.tail, W);                     // without FAST: see the checkpoint sweep
    const bool lastm = b == p.Bt - 1;
    bool lastB[NW];
#pragma unroll
    for (int s = 0; s < NW; ++s) lastB[s] = lastm && (n0 + (s < nvalid ? s : 0) == N - 1);
    const int nv = FAST ? (inside ? K : 0) : max(0, min(K, W - col0));   // cells of this lane inside the map
    const uint8_t* mm = p.mask ? p.mask + (size_t)b * HW : nullptr;
    const T* Bs[NW];
    const T* Cs[NW];
#pragma unroll
    for (int s = 0; s < NW; ++s) {
        const int n = n0 + (s < nvalid ? s : 0);
        Bs[s] = reinterpret_cast<const T*>(p.Bm) + ((size_t)b * N + n) * HW;
        Cs[s] = reinterpret_cast<const T*>(p.Cm) + ((size_t)b * N + n) * HW;
    }

    for (int ch = 0; ch < GS; ++ch) {
#pragma unroll
        for (int e = 0; e < NW * K; ++e) gaL[((size_t)ch * THREADS + tid) * (NW * K) + e] = 0.0f;   // g below the map is 0
#pragma unroll
        for (int s = 0; s < NW; ++s) dAL[((size_t)ch * THREADS + tid) * NW + s] = 0.0f;
        dDL[(size_t)ch * THREADS + tid] = 0.0f;
    }
    // every thread only ever touches its own gaL / dAL / dDL entries: no barrier needed for them

    int step = 0;                                         // rows reduced so far: parity picks the LDS buffer
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
            const bool lastx = map == (size_t)p.Bt * p.Dc - 1;
            const T* xm = reinterpret_cast<const T*>(p.x) + map * HW;
            const DT* dm = reinterpret_cast<const DT*>(p.delta) + map * HW;
            float* ddw = SP ? const_cast<float*>(reinterpret_cast<const float*>(p.delta)) + map * HW : nullptr;
            const T* dym = reinterpret_cast<const T*>(p.dy) + map * HW;
            T* dxm = reinterpret_cast<T*>(p.dx) + map * HW;
            T* ddm = reinterpret_cast<T*>(p.ddelta) + map * HW;
            float An[NW], Ap[NW], Avn[NW], Avp[NW];
#pragma unroll
            for (int s = 0; s < NW; ++s) {
                An[s] = p.A[(size_t)c * N + n0 + (s < nvalid ? s : 0)];
                Ap[s] = An[s] * kLog2e;
                Avn[s] = AV ? p.A_v[(size_t)c * N + n0 + (s < nvalid ? s : 0)] : 0.0f;
                Avp[s] = Avn[s] * kLog2e;
            }
            const float dsk = (p.Dskip != nullptr && sg == 0) ? p.Dskip[c] : 0.0f;

            // ---- scans 1 and 2: rebuild h[i-1,j] and hhor[i,j-1] for the rows of the band
            float hprev[RB][NW][K], hhl[RB][NW][K];
            if (act) {
                uint32_t fx[2][XW], fd[2][XWD], fm[2][K / 4], fB[2][NW][XW];
                auto issue = [&](int buf, int i) {
                    const size_t ro = (size_t)i * W;
                    const bool bottom = i == H - 1;
                    ld_elems<T, K, FAST>(xm + ro, lcol, lastx && bottom, tl.x, fx[buf]);
                    ld_elems<DT, K, FAST>(dm + ro, lcol, !SP && lastx && bottom, reinterpret_cast<const DT*>(tl.delta), fd[buf]);
                    ld_mask<K, FAST>(mm ? mm + ro : nullptr, lcol, lastm && bottom, tl.mask, fm[buf]);
#pragma unroll
                    for (int s = 0; s < NW; ++s) ld_elems<T, K, FAST>(Bs[s] + ro, lcol, lastB[s] && bottom, tl.B, fB[buf][s]);
                };
                if constexpr (PF) issue(0, r0);
                float hcur[NW][K];
#pragma unroll
                for (int s = 0; s < NW; ++s) {
                    const float* src = p.ck + ((map * p.nb + band) * N + n0 + (s < nvalid ? s : 0)) * W;
                    if (band == 0) {
#pragma unroll
                        for (int j = 0; j < K; ++j) hcur[s][j] = 0.0f;
                    } else {
                        load_f32s<K>(src + lcol, hcur[s]);               // past the row end: the next checkpoint row or the region behind
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
                        else issue(r & 1, i);
                        float dl[K], dxe[K];
#pragma unroll
                        for (int j = 0; j < K; ++j) {
                            dl[j] = get_elem<DT, K>(fd[r & 1], j);
                            if (SP && !FAST && j >= nv) dl[j] = 0.0f;     // past the row end: the row below already holds gradients
                            // past the row end x belongs to the next map but the mask bytes to the next batch item: no x there
                            const float xe = (mask_bit<K>(fm[r & 1], j) || (!FAST && j >= nv)) ? 0.0f : get_elem<T, K>(fx[r & 1], j);
                            dxe[j] = dl[j] * xe;
                        }
#pragma unroll
                        for (int s = 0; s < NW; ++s) {
                            float a[K], hl[K], pl[K];
#pragma unroll
                            for (int j = 0; j < K; ++j) a[j] = __builtin_amdgcn_exp2f(dl[j] * Ap[s]);
                            hl[0] = dxe[0] * get_elem<T, K>(fB[r & 1][s], 0);
                            pl[0] = a[0];
                            float hcv = 0.0f;                             // state entering from the panel to the left
                            if (p.hc_in != nullptr && l == 0) {
                                hcv = p.hc_in[(map * N + n0 + (s < nvalid ? s : 0)) * H + i];
                                hl[0] = fmaf(a[0], hcv, hl[0]);
                            }
#pragma unroll
                            for (int j = 1; j < K; ++j) {
                                hl[j] = fmaf(a[j], hl[j - 1], dxe[j] * get_elem<T, K>(fB[r & 1][s], j));
                                pl[j] = pl[j - 1] * a[j];
                            }
                            float P[1] = {pl[K - 1]}, Hh[1] = {hl[K - 1]}, cin[1];
                            group_scan<LG, 1>(P, Hh, cin);
                            float left = cin[0];                          // hhor[i, j-1]
                            if (p.hc_in != nullptr && l == 0) left = hcv;
#pragma unroll
                            for (int j = 0; j < K; ++j) {
                                const float hh = (j == K - 1) ? Hh[0] : fmaf(pl[j], cin[0], hl[j]);
                                hhl[r][s][j] = left;
                                hprev[r][s][j] = hcur[s][j];
                                if constexpr (AV) hcur[s][j] = fmaf(__builtin_amdgcn_exp2f(dl[j] * Avp[s]), hcur[s][j], hh);
                                else fma_inplace(hcur[s][j], a[j], hh);
                                left = hh;
                            }
                        }
                    }
                }
            }

            // ---- scans 3 and 4, bottom row of the band first
            float ga[NW][K], dAb[NW], dVb[NW], dDb = 0.0f;
#pragma unroll
            for (int s = 0; s < NW; ++s) {
                dAb[s] = 0.0f;
                dVb[s] = 0.0f;
#pragma unroll
                for (int j = 0; j < K; ++j) ga[s][j] = gaL[((size_t)ch * THREADS + tid) * (NW * K) + s * K + j];
            }
            uint32_t bx[2][XW], bd[2][XWD], by[2][XW], bm[2][K / 4], bB[2][NW][XW], bC[2][NW][XW];
            auto issue_r = [&](int buf, int i) {
                const size_t ro = (size_t)i * W;
                const bool bottom = i == H - 1;
                ld_elems<T, K, FAST>(xm + ro, lcol, lastx && bottom, tl.x, bx[buf]);
                ld_elems<DT, K, FAST>(dm + ro, lcol, !SP && lastx && bottom, reinterpret_cast<const DT*>(tl.delta), bd[buf]);
                ld_elems<T, K, FAST>(dym + ro, lcol, lastx && bottom, tl.dy, by[buf]);
                ld_mask<K, FAST>(mm ? mm + ro : nullptr, lcol, lastm && bottom, tl.mask, bm[buf]);
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
                        issue_r(r & 1, i);
                    }
                    const size_t ro = (size_t)i * W;
                    float dl[K], xe[K], dxe[K], dyv[K], ddl[K], dxl[K];
#pragma unroll
                    for (int j = 0; j < K; ++j) {
                        dl[j] = get_elem<DT, K>(bd[r & 1], j);
                        if (SP && !FAST && j >= nv) dl[j] = 0.0f;
                        xe[j] = (mask_bit<K>(bm[r & 1], j) || (!FAST && j >= nv)) ? 0.0f : get_elem<T, K>(bx[r & 1], j);
                        dxe[j] = dl[j] * xe[j];
                        dyv[j] = get_elem<T, K>(by[r & 1], j);
                        if (FAST ? !inside : j >= nv) dyv[j] = 0.0f;      // nothing flows out of a cell past the map
                        ddl[j] = 0.0f;
                        dxl[j] = dsk * dyv[j];
                        dDb = fmaf(dyv[j], xe[j], dDb);
                    }
#pragma unroll
                    for (int s = 0; s < NW; ++s) {
                        if (act && s < nvalid) {
                            float a[K], av[K], Bv[K], g[K];
#pragma unroll
                            for (int j = 0; j < K; ++j) {
                                a[j] = __builtin_amdgcn_exp2f(dl[j] * Ap[s]);
                                av[j] = AV ? __builtin_amdgcn_exp2f(dl[j] * Avp[s]) : a[j];
                                Bv[j] = get_elem<T, K>(bB[r & 1][s], j);
                                const float hh = fmaf(a[j], hhl[r][s][j], dxe[j] * Bv[j]);   // hhor[i,j]
                                const float hv = fmaf(av[j], hprev[r][s][j], hh);            // h[i,j]
                                dCacc[r][s][j] = fmaf(dyv[j], hv, dCacc[r][s][j]);
                                g[j] = fmaf(dyv[j], get_elem<T, K>(bC[r & 1][s], j), ga[s][j]);   // scan 3
                                ga[s][j] = av[j] * g[j];
                            }
                            // scan 4: q[j] = g[j] + a[j+1] * q[j+1]
                            float ar[K], ql[K], pr[K];
#pragma unroll
                            for (int j = 0; j + 1 < K; ++j) ar[j] = a[j + 1];
                            ar[K - 1] = from_right<LG>(a[0]);
                            ql[K - 1] = g[K - 1];
                            if (p.qc_in != nullptr && l == LG - 1)        // a*q entering from the panel to the right
                                ql[K - 1] += p.qc_in[(map * N + n0 + s) * H + i];
                            pr[K - 1] = ar[K - 1];
#pragma unroll
                            for (int j = K - 2; j >= 0; --j) {
                                ql[j] = fmaf(ar[j], ql[j + 1], g[j]);
                                pr[j] = ar[j] * pr[j + 1];
                            }
                            float P[1] = {pr[0]}, Q[1] = {ql[0]}, qin[1];
                            group_scan_left<LG, 1>(P, Q, qin);
#pragma unroll
                            for (int j = 0; j < K; ++j) {
                                const float q = fmaf(pr[j], qin[0], ql[j]);
                                if (j == 0 && p.qc_out != nullptr && l == 0) p.qc_out[(map * N + n0 + s) * H + i] = a[0] * q;
                                if constexpr (AV) {
                                    const float th = q * hhl[r][s][j] * a[j];                // through the row recurrence's decay
                                    const float tv = g[j] * hprev[r][s][j] * av[j];          // through the column recurrence's decay
                                    dAb[s] = fmaf(th, dl[j], dAb[s]);
                                    dVb[s] = fmaf(tv, dl[j], dVb[s]);
                                    ddl[j] = fmaf(th, An[s], fmaf(tv, Avn[s], fmaf(q * Bv[j], xe[j], ddl[j])));
                                } else {
                                const float da = fmaf(g[j], hprev[r][s][j], q * hhl[r][s][j]);
                                const float t = da * a[j];
                                dAb[s] = fmaf(t, dl[j], dAb[s]);
                                ddl[j] = fmaf(t, An[s], fmaf(q * Bv[j], xe[j], ddl[j]));
                                }
                                dxl[j] = fmaf(q * dl[j], Bv[j], dxl[j]);
                                dBacc[r][s][j] = fmaf(q, dxe[j], dBacc[r][s][j]);
                            }
                        }
                    }
                    // sums over the states held by the other lane groups of this map
                    float* mine = part + (size_t)(step & 1) * 2 * THREADS * K + (size_t)tid * K;
#pragma unroll
                    for (int j = 0; j < K; ++j) {
                        mine[j] = ddl[j];
                        mine[THREADS * K + j] = mask_bit<K>(bm[r & 1], j) ? 0.0f : dxl[j];
                    }
                    __syncthreads();
                    if (act) {
                        const float* base = part + (size_t)(step & 1) * 2 * THREADS * K + (size_t)(slot - sg) * PANEL;
                        for (int col = sg * LG + l; col < PANEL; col += NG * LG) {
                            const int gc = p.cb + col;
                            if (gc < W) {
                                const float dd = sum_partials<PANEL>(base + col, NG);
                                if constexpr (SP) ddw[ro + gc] = dd;        // over the step of this cell, which nobody reads again
                                else store_elem(ddm + ro + gc, dd);
                                store_elem(dxm + ro + gc, sum_partials<PANEL>(base + THREADS * K + col, NG));
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
                dAL[((size_t)ch * THREADS + tid) * NW + s] += inside ? dAb[s] : 0.0f;
                if constexpr (AV) dVtot[s] += inside ? dVb[s] : 0.0f;
            }
            dDL[(size_t)ch * THREADS + tid] += dDb;
        }

        // partial sums over this workgroup's channels, one write per band
        if (live) {
#pragma unroll
            for (int r = 0; r < RB; ++r) {
                const int i = r0 + r;
                if (i < H) {
#pragma unroll
                    for (int s = 0; s < NW; ++s) {
                        if (s < nvalid) {
                            const size_t o = ((((size_t)b * p.CG + cg) * N + n0 + s) * H + i) * W;
                            if (nv == K) {
                                store_f32s<K>(p.pB + o + col0, dBacc[r][s]);
                                store_f32s<K>(p.pC + o + col0, dCacc[r][s]);
                            } else if (!FAST) {
#pragma unroll
                                for (int j = 0; j < K; ++j)
                                    if (col0 + j < W) { p.pB[o + col0 + j] = dBacc[r][s][j]; p.pC[o + col0 + j] = dCacc[r][s][j]; }
                            }
                        }
                    }
                }
            }
        }
    }

    if constexpr (AV) {                               // dA_v[b,c,n], summed like dA below
        for (int ch = 0; ch < GS; ++ch) {
            const bool act = ch < nch;
            const int c = c_first + ch;
#pragma unroll
            for (int s = 0; s < NW; ++s) {
                float v = row_sum16(dVtot[s]);
                if constexpr (LG == 64) {
                    const int vi = __builtin_bit_cast(int, v);
                    v = __builtin_bit_cast(float, __builtin_amdgcn_readlane(vi, 0)) +
                        __builtin_bit_cast(float, __builtin_amdgcn_readlane(vi, 16)) +
                        __builtin_bit_cast(float, __builtin_amdgcn_readlane(vi, 32)) +
                        __builtin_bit_cast(float, __builtin_amdgcn_readlane(vi, 48));
                }
                if (act && l == 0 && s < nvalid) {
                    float* dst = p.pAv + ((size_t)b * p.Dc + c) * N + n0 + s;
                    *dst = p.accum ? *dst + v : v;
                }
            }
        }
    }
    // dA[b,c,n] and dDskip[b,c]: sum the per-lane partials over the lane group in a fixed order
    for (int ch = 0; ch < GS; ++ch) {                 // uniform trip count: the sums use DPP
        const bool act = ch < nch;
        const int c = c_first + ch;
#pragma unroll
        for (int s = 0; s <= NW; ++s) {               // s == NW: the dDskip partial
            float v = (s < NW) ? dAL[((size_t)ch * THREADS + tid) * NW + (s < NW ? s : 0)]
                               : dDL[(size_t)ch * THREADS + tid];
            v = row_sum16(v);
            if constexpr (LG == 64) {
                const int vi = __builtin_bit_cast(int, v);
                v = __builtin_bit_cast(float, __builtin_amdgcn_readlane(vi, 0)) +
                    __builtin_bit_cast(float, __builtin_amdgcn_readlane(vi, 16)) +
                    __builtin_bit_cast(float, __builtin_amdgcn_readlane(vi, 32)) +
                    __builtin_bit_cast(float, __builtin_amdgcn_readlane(vi, 48));
            }
            if (act && l == 0) {
                if (s < NW) {
                    if (s < nvalid) {
                        float* dst = p.pA + ((size_t)b * p.Dc + c) * N + n0 + s;
                        *dst = p.accum ? *dst + v : v;            // panels are launched one after the other
                    }
                } else if (sg == 0 && p.pD != nullptr) {
                    float* dst = p.pD + (size_t)b * p.Dc + c;
                    *dst = p.accum ? *dst + v : v;
                }
            }
        }
    }
}

}  // namespace scan2d
