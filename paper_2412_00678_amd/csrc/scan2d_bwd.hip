// Host side of the backward pass: variant choice, workspace layout, launches.
#include "scan2d_bwd.hpp"

#include <algorithm>
#include <cstdio>
#include <cstdlib>

#include "scan2d_bwd_variants.hpp"
#include "scan2d_tuning.hpp"

namespace scan2d {
namespace {

// ------------------------------------------------------------------------------ final sums
// dBm/dCm[b,n,i,j] = sum over channel groups of the partials; one thread per element.
__global__ void scan2d_bwd_reduce_groups_kernel(const float* __restrict__ pB, const float* __restrict__ pC,
                                                float* __restrict__ dBm, float* __restrict__ dCm,
                                                int Bt, int CG, size_t NHW) {
    const size_t total = (size_t)Bt * NHW;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
        const size_t b = e / NHW, r = e - b * NHW;
        const float* sB = pB + b * CG * NHW + r;
        const float* sC = pC + b * CG * NHW + r;
        float aB = 0.0f, aC = 0.0f;
        for (int g = 0; g < CG; ++g) { aB += sB[(size_t)g * NHW]; aC += sC[(size_t)g * NHW]; }
        dBm[e] = aB;
        dCm[e] = aC;
    }
}

// The same sum for partials whose rows are LG*K floats in the lane order of the main sweep, [K/4][LG][4]: element q of a
// row is column (q / 4 % LG) * K + (q / (4 * LG)) * 4 + q % 4.  rows = N * H.
__global__ void scan2d_bwd_reduce_groups_chunked_kernel(const float* __restrict__ pB, const float* __restrict__ pC,
                                                        float* __restrict__ dBm, float* __restrict__ dCm,
                                                        int Bt, int CG, size_t rows, int W, int LG, int K) {
    const size_t panel = (size_t)LG * K, per_item = rows * panel, total = (size_t)Bt * per_item;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
        const size_t b = e / per_item, r = e - b * per_item;
        const size_t row = r / panel;
        const int q = (int)(r - row * panel);
        const int col = (q / 4 % LG) * K + (q / (4 * LG)) * 4 + q % 4;
        if (col >= W) continue;
        const float* sB = pB + b * CG * per_item + r;
        const float* sC = pC + b * CG * per_item + r;
        float aB = 0.0f, aC = 0.0f;
        for (int g = 0; g < CG; ++g) { aB += sB[(size_t)g * per_item]; aC += sC[(size_t)g * per_item]; }
        const size_t o = (b * rows + row) * W + col;
        dBm[o] = aB;
        dCm[o] = aC;
    }
}

// dA[c,n] = sum_b pA[b,c,n]; dDskip[c] = sum_b pD[b,c].
__global__ void scan2d_bwd_reduce_batch_kernel(const float* __restrict__ pA, const float* __restrict__ pD,
                                               float* __restrict__ dA, float* __restrict__ dDskip,
                                               int Bt, int Dc, int N) {
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < Dc * N) {
        float acc = 0.0f;
        for (int b = 0; b < Bt; ++b) acc += pA[(size_t)b * Dc * N + e];
        dA[e] = acc;
    }
    if (dDskip != nullptr && e < Dc) {
        float acc = 0.0f;
        for (int b = 0; b < Bt; ++b) acc += pD[(size_t)b * Dc + e];
        dDskip[e] = acc;
    }
}

// ddelta_bias: per map, the sum of the (already chain-ruled) ddelta_raw over positions, in a fixed
// order (strided partial sums per thread, then a tree over the workgroup); summed over batch items
// by scan2d_bwd_reduce_bias_batch_kernel.
template <typename T>
__global__ __launch_bounds__(256) void scan2d_bwd_reduce_bias_kernel(const T* __restrict__ ddelta_raw, float* __restrict__ pbias, size_t HW) {
    __shared__ float sh[256];
    const T* src = ddelta_raw + (size_t)blockIdx.x * HW;
    float acc = 0.0f;
    for (size_t e = threadIdx.x; e < HW; e += 256) {
        if constexpr (Elem<T>::kBytes == 4) acc += __uint_as_float(elem_bits(src + e));
        else acc += __uint_as_float(elem_bits(src + e) << 16);
    }
    sh[threadIdx.x] = acc;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) sh[threadIdx.x] += sh[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) pbias[blockIdx.x] = sh[0];
}
__global__ void scan2d_bwd_reduce_bias_batch_kernel(const float* __restrict__ pbias, float* __restrict__ dbias, int Bt, int Dc) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c < Dc) {
        float acc = 0.0f;
        for (int b = 0; b < Bt; ++b) acc += pbias[(size_t)b * Dc + c];
        dbias[c] = acc;
    }
}

// Softplus step, banded form: the step is computed once per position here, as fp32 whatever the storage
// type, instead of by each of a map's lane groups in both sweeps (16-fold in the main sweep for N = 16: a
// fifth of its run time); the SP instantiations of the sweeps read it.  One workgroup per 1024 positions of
// a map (`chunks` per map).
template <typename T>
__global__ __launch_bounds__(256) void scan2d_bwd_step_kernel(const T* __restrict__ raw, const float* __restrict__ bias,
                                                              float* __restrict__ step, size_t HW, int Dc, unsigned chunks) {
    const size_t map = blockIdx.x / chunks;
    const float b = bias != nullptr ? bias[map % Dc] : 0.0f;
    const T* src = raw + map * HW;
    float* dst = step + map * HW;
    const size_t e0 = ((size_t)(blockIdx.x % chunks) * 256 + threadIdx.x) * 4;
    if (e0 + 4 <= HW && (Elem<T>::kBytes == 4 || (HW & 1) == 0)) {      // four elements at once (rows of a map stay 4-byte aligned)
        uint32_t r[words_of<T, 4>()], o[4];
        load_words<words_of<T, 4>()>(reinterpret_cast<const uint32_t*>(src + e0), r);
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = __float_as_uint(softplus_f32(get_elem<T, 4>(r, j) + b));
        store_words<4>(reinterpret_cast<uint32_t*>(dst + e0), o);
        return;
    }
    for (size_t e = e0; e < e0 + 4 && e < HW; ++e) {
        float t;
        if constexpr (Elem<T>::kBytes == 4) t = __uint_as_float(elem_bits(src + e));
        else t = __uint_as_float(elem_bits(src + e) << 16);
        dst[e] = softplus_f32(t + b);
    }
}

// The matching chain rule: `dstep` (fp32, the gradient of the step as the main sweep left it in the workspace)
// becomes the gradient of the raw projection, ddelta_raw = dstep / (1 + exp(-(raw + bias))), rounded once to
// the storage type; its sum over the map's positions, taken from the stored values, goes to pbias (null: no
// bias) in a fixed order (strided partial sums per thread, then a tree over the workgroup).
template <typename T>
__global__ __launch_bounds__(256) void scan2d_bwd_chain_kernel(const float* __restrict__ dstep, const T* __restrict__ raw,
                                                               const float* __restrict__ bias, T* __restrict__ ddelta_raw,
                                                               float* __restrict__ pbias, size_t HW, int Dc) {
    __shared__ float sh[256];
    const size_t map = blockIdx.x;
    const float b = bias != nullptr ? bias[map % Dc] : 0.0f;
    const float* dd = dstep + map * HW;
    const T* src = raw + map * HW;
    T* dst = ddelta_raw + map * HW;
    float acc = 0.0f;
    for (size_t e = threadIdx.x; e < HW; e += 256) {
        float t;
        if constexpr (Elem<T>::kBytes == 4) t = __uint_as_float(elem_bits(src + e));
        else t = __uint_as_float(elem_bits(src + e) << 16);
        const float v = dd[e] * logistic_f32(t + b);
        store_elem(dst + e, v);
        if constexpr (Elem<T>::kBytes == 4) acc += v;
        else acc += __uint_as_float(f32_to_bf16_bits(v) << 16);
    }
    if (pbias == nullptr) return;                        // uniform over the grid
    sh[threadIdx.x] = acc;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) sh[threadIdx.x] += sh[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) pbias[map] = sh[0];
}

// Padded copies of the rows behind which the input tensors end (layout: TailRows in scan2d_bwd_kernels.hpp):
// the last row of the last map of x, delta and dy, of the last state plane of Bm and Cm, and of the last
// batch item's mask, each followed by 16 zeros.  The instantiations for widths that are not a multiple of
// the columns per lane read these rows from here, because their last lane reads past the end of a row.
template <typename T>
__global__ __launch_bounds__(256) void scan2d_bwd_tail_kernel(const T* __restrict__ x, const T* __restrict__ delta, const T* __restrict__ dy,
                                                              const T* __restrict__ Bm, const T* __restrict__ Cm,
                                                              const uint8_t* __restrict__ mask, T* __restrict__ tail,
                                                              size_t last_map_row, size_t last_plane_row, size_t last_mask_row, int W) {
    const int ts = W + 16;
    uint8_t* tm = reinterpret_cast<uint8_t*>(tail + 5 * (size_t)ts);
    for (int j = threadIdx.x; j < ts; j += 256) {
        const bool in = j < W;
        T zero;
        if constexpr (Elem<T>::kBytes == 4) zero = 0.0f; else zero.bits = 0;
        tail[j] = in ? x[last_map_row + j] : zero;
        tail[ts + j] = in ? delta[last_map_row + j] : zero;
        tail[2 * (size_t)ts + j] = in ? dy[last_map_row + j] : zero;
        tail[3 * (size_t)ts + j] = in ? Bm[last_plane_row + j] : zero;
        tail[4 * (size_t)ts + j] = in ? Cm[last_plane_row + j] : zero;
        tm[j] = (in && mask != nullptr) ? mask[last_mask_row + j] : (uint8_t)0;
    }
}

struct BwdPlan {
    bool small = false;                                    // one wavefront per map, no bands (scan2d_bwd_small.hpp)
    int LG = 0, K = 0, NW = 0, waves = 0, RB = 0;
    int NG = 0, GS = 0, CG = 0, nb = 0;
    BwdKernels k;
    size_t lds_bytes = 0;
    int panels = 1;                                        // column panels of LG*K columns, one launch of each sweep per panel
    size_t off_hc = 0, off_qc = 0;                         // carries between panels: [panels-1][maps][N][H] and [2][maps][N][H]
    bool shared = false;                                   // main sweep of scan2d_bwd_shared.hpp
    int ck_LG = 0, ck_waves = 0;                           // lane tiling of the checkpoint sweep
    bool step_outside = false;                             // softplus step written by a kernel of its own (banded form)
    size_t off_step = 0;                                   // the step [maps][H][W] fp32 (step_outside only), 256 spare bytes behind it
    bool fast = true;                                      // W is a multiple of the columns per lane
    size_t off_tail = 0;                                   // padded copies of the tensors' last rows (TailRows)
    size_t off_ck = 0, off_pB = 0, off_pC = 0, off_pA = 0, off_pD = 0, off_pb = 0, total = 0;   // pb: bias-gradient partials
    bool av = false;                                       // independent decay of the column recurrence
    bool ck_chunked = false;                               // checkpoint rows in the lane order of the two shared-producer sweeps
    bool part_chunked = false;                             // rows of the dBm / dCm partials in the lane order of the main sweep
    size_t off_pAv = 0;                                    // partial sums of dA_v over batch items
};

size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

// Tilings whose shared-producer main sweep is the default: measured 10-30 % faster than the plain one for 16-lane
// groups (56x56 bf16 x 6144 maps: 1.41 -> 1.08 ms; 128x192 fp32 x 2048 maps: 3.63 -> 2.86 ms); slower for wave-wide
// groups on 16 waves, where the 128-register budget makes it spill (256x256 bf16: 2.0 -> 3.0 ms).
bool shared_by_default(int LG, int K, int NW) { return LG == 16 || (LG == 64 && K == 4 && NW == 2); }

}  // namespace
bool allow_large_lds(const void* kernel, size_t bytes);   // scan2d_api.hip
namespace {

bool make_plan(const scan2d_desc* d, BwdPlan* out, bool sp = false, bool av = false) {
    BwdPlan pl;
    pl.av = av;
    const int W = d->W, N = d->N;
    // columns first inside the kernels: only the banded form with the shared-producer main sweep has such
    // instantiations; no plan otherwise (the caller then runs columns first through transposes)
    const bool cf = (d->flags & SCAN2D_FLAG_COLUMNS_FIRST) != 0;
    if (cf && av) return false;
    const TuneValues tb = av ? TuneValues() : tune_get(kTuneBwd);
    if (W <= 16 && d->H <= 16 && N <= 16 && tb.n == 0 && !av && !cf) {
        // small maps: the whole map stays in registers; dBm/dCm partials per channel
        pl.small = true;
        pl.LG = 16; pl.K = 1; pl.NW = N <= 4 ? 1 : (N <= 8 ? 2 : 4); pl.waves = 4; pl.RB = d->H;
        pl.NG = 4; pl.GS = 1; pl.CG = d->Dc; pl.nb = 1; pl.lds_bytes = 0;
        pl.k.main = d->dtype == SCAN2D_BF16 ? bwd_small_kernel_bf16(pl.NW, sp) : bwd_small_kernel_f32(pl.NW, sp);
        if (pl.k.main == nullptr) return false;
        const size_t maps = (size_t)d->Bt * d->Dc;
        const size_t NHW = (size_t)N * d->H * W;
        size_t o = 0;
        pl.off_ck = o;
        pl.off_pB = o; o += pl.CG > 1 ? align_up(maps * NHW * sizeof(float)) : 0;
        pl.off_pC = o; o += pl.CG > 1 ? align_up(maps * NHW * sizeof(float)) : 0;
        pl.off_pA = o; o += d->Bt > 1 ? align_up(maps * N * sizeof(float)) : 0;
        pl.off_pD = o; o += d->Bt > 1 ? align_up(maps * sizeof(float)) : 0;
        pl.off_pb = o; o += align_up(maps * sizeof(float));
        pl.total = o;
        *out = pl;
        return true;
    }
    int LG, K;
    if (W <= 64) { LG = 16; K = 4; }
    else if (W <= 128) { LG = 16; K = 8; }
    else if (W <= 192 && N <= 16) { LG = 16; K = 12; }         // 12 columns x 4 states per lane would not fit the registers
    else if (W <= 256) { LG = 64; K = 4; }
    else if (W <= 512) { LG = 64; K = 8; }
    else if (W <= 1024) { LG = 64; K = 16; }
    else { LG = 64; K = 4; }
    // maps wider than the widest tiling (and, beyond 16 states, wider than 256 columns: the band arrays of four
    // states per lane and 16 waves fill the LDS) are swept in panels of 256 columns
    // (measured faster than the 8- and 16-column tilings from 257 columns on: 512x512 bf16 x 256 maps 9.97 -> 8.74 ms)
    if (W > 256 || av) { LG = 64; K = 4; pl.panels = (W + 255) / 256; }
    int force_waves = 0, force_gs = 0, want_shared = -1;
    if (tb.n >= 1) {                                             // tuning aid: LG,K[,WAVES[,GS[,shared]]]
        const int eLG = tb.v[0], eK = tb.v[1], eW = tb.v[2], eG = tb.v[3];
        const int got = tb.n;
        if (got >= 2 && (eLG == 16 || eLG == 32 || eLG == 64) && eLG * eK >= W && W <= 1024 && (N <= 16 || W <= 256)) {
            LG = eLG; K = eK; pl.panels = 1;                     // a single-panel tiling forced on a map it covers
        }
        if (got >= 3) force_waves = eW;
        if (got >= 4) force_gs = eG;
        if (got >= 5) want_shared = tb.v[4];
    }
    // states per lane and waves per workgroup: 16 lane groups of one DPP row with one state each;
    // wavefront-wide lane groups: 16 of them with one state each for 4 columns per lane (four waves
    // per SIMD: measured 20-30 % faster than 8 groups of two states), 8 with two states each for 8
    // columns; four states per lane beyond N = 16
    int waves, NW;
    if (LG == 16) { waves = 4; NW = N <= 16 ? 1 : 4; }
    else if (LG == 32) { waves = 8; NW = 1; }
    else if (N <= 16 && K == 16) { waves = 4; NW = 4; }     // widest maps: LDS bounds the workgroup size
    // (one panel of 16 states: two states per lane on 8 waves with the shared-producer main sweep, measured 13 % faster
    // than 16 waves of one state that each repeat the per-position work: 256 maps of 256x256 bf16 2.11 -> 1.83 ms)
    else if (N == 16 && K == 4 && !av && want_shared != 0 && force_waves != 16) { waves = 8; NW = 2; }
    else if (N <= 16 && K == 4 && force_waves != 8) { waves = 16; NW = 1; }
    else if (N <= 16) { waves = 8; NW = 2; }
    else { waves = 16; NW = 4; }
    const int slots = waves * 64 / LG;
    if ((N + NW - 1) / NW > slots) return false;
    const bool fast = (W % K) == 0;                          // otherwise: the instantiations that treat the row end
    pl.step_outside = sp;
    pl.fast = fast;
    // the main sweep that shares the per-position work through LDS, where it exists for this tiling (N = NG * NW)
    if (want_shared != 0 && N % NW == 0 && !av) {              // (its kernels take column panels too)
        BwdKernels ks;
        if (cf) ks = d->dtype == SCAN2D_BF16 ? bwd_shared_kernels_bf16_cf(LG, K, NW, N / NW, waves, W, sp)
                                             : bwd_shared_kernels_f32_cf(LG, K, NW, N / NW, waves, W, sp);
        else ks = d->dtype == SCAN2D_BF16 ? bwd_shared_kernels_bf16(LG, K, NW, N / NW, waves, W, sp)
                                          : bwd_shared_kernels_f32(LG, K, NW, N / NW, waves, W, sp);
        if (pl.panels > 1) ks.main = ks.main_panels;              // column panels: the instantiation that takes them, if any
        if (ks.main != nullptr && (want_shared == 1 || shared_by_default(LG, K, NW))) pl.k = ks;
    }
    if (cf && pl.k.main == nullptr) return false;
    if (av) {
        if (sp) return false;
        pl.k = d->dtype == SCAN2D_BF16 ? bwd_kernels_av_bf16(NW, fast) : bwd_kernels_av_f32(NW, fast);
    }
    if (pl.k.main == nullptr)
        pl.k = d->dtype == SCAN2D_BF16 ? bwd_kernels_bf16(LG, K, NW, waves, fast, sp) : bwd_kernels_f32(LG, K, NW, waves, fast, sp);
    if (pl.k.main == nullptr) return false;
    pl.shared = pl.k.shared;
    // the single-panel shared-producer sweeps apply the softplus and its chain rule themselves (their checkpoint sweep,
    // the shared-producer forward kernel, computes the step from the raw projection too)
    if (pl.shared && pl.panels == 1 && pl.k.ckpt_fwd != nullptr && N == pl.k.cf_NG * pl.k.cf_NW) pl.step_outside = false;
    pl.fast = fast && pl.k.ckpt_fast;                        // false: the padded copies of the tensors' last rows are needed
    pl.ck_LG = pl.k.ckpt_LG; pl.ck_waves = pl.k.ckpt_waves;
    pl.LG = LG; pl.K = K; pl.NW = NW; pl.waves = waves; pl.RB = pl.k.RB;
    pl.NG = (N + NW - 1) / NW;
    pl.nb = (d->H + pl.RB - 1) / pl.RB;
    // channels a workgroup handles one after the other: bounded by the 160 KB of LDS; among the
    // feasible counts take the one with the shortest critical path (rounds of resident workgroups
    // - the runtime's occupancy figure for the kernel's registers and this much LDS, one per CU
    // if it cannot be asked - times channels per workgroup), the larger count on a tie (fewer
    // partial sums to write and add up)
    const size_t T = (size_t)waves * 64;
    size_t fixed = 4 * T * K, per = T * ((size_t)NW * K + NW + 1);
    if (pl.shared) {             // see the LDS layout in scan2d_bwd_shared.hpp
        fixed = 4 * T * K + (T / (size_t)pl.NG / LG) * ((size_t)pl.RB * 5 * LG * K);
        per = T * (size_t)NW * K + (T / LG) * NW + (size_t)waves;
        if (sp && !pl.step_outside) per += (size_t)waves;     // the bias gradient per wavefront
    }
    const int gs_lds = (int)std::max<size_t>(1, (40960 - std::min<size_t>(fixed, 40960)) / per);
    const int JPW = slots / pl.NG;
    const int gs_max = av ? 1 : std::min({gs_lds, 8, d->Dc});   // av: one channel per workgroup (its dA_v partial stays in registers)
    int gs = 1;
    long long best_path = -1;
    for (int g = 1; g <= gs_max; ++g) {
        const long long jobs = (long long)d->Bt * ((d->Dc + g - 1) / g);
        const long long wgs = (jobs + JPW - 1) / JPW;
        int per_cu = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(pl.k.main), (int)T,
                                                         (fixed + (size_t)g * per) * sizeof(float)) != hipSuccess || per_cu < 1) {
            (void)hipGetLastError();
            per_cu = 1;
        }
        const long long resident = 256LL * per_cu;
        const long long path = ((wgs + resident - 1) / resident) * g;
        if (best_path < 0 || path <= best_path) { best_path = path; gs = g; }
    }
    if (force_gs >= 1 && force_gs <= gs_lds && force_gs <= d->Dc) gs = force_gs;
    pl.GS = gs;
    pl.CG = (d->Dc + gs - 1) / gs;
    pl.lds_bytes = (fixed + (size_t)gs * per) * sizeof(float);
    if (pl.lds_bytes > 160 * 1024) return false;
    const size_t maps = (size_t)d->Bt * d->Dc;
    size_t o = 0;
    // the shared-producer forward kernel writes the checkpoints and the shared-producer main sweep reads them with the same
    // lane tiling: rows of LG*K floats in lane order, so that both move whole 16-byte x LG pieces per instruction
    // (only where the padding of the rows to LG*K columns costs less than 7 %)
    const bool tight = (size_t)LG * K * 15 <= (size_t)W * 16;
    pl.ck_chunked = tight && pl.shared && pl.panels == 1 && pl.k.ckpt_fwd != nullptr && N == pl.k.cf_NG * pl.k.cf_NW && pl.k.cf_LG == LG &&
                    pl.k.cf_K == K && K % 4 == 0;
    pl.off_ck = o; o += align_up(maps * pl.nb * N * (pl.ck_chunked ? (size_t)LG * K : (size_t)W) * sizeof(float));
    pl.part_chunked = tight && pl.shared && pl.panels == 1 && pl.CG > 1 && K % 4 == 0;
    const size_t part_row = pl.part_chunked ? (size_t)LG * K : (size_t)W;
    pl.off_pB = o; o += pl.CG > 1 ? align_up((size_t)d->Bt * pl.CG * N * d->H * part_row * sizeof(float)) : 0;
    pl.off_pC = o; o += pl.CG > 1 ? align_up((size_t)d->Bt * pl.CG * N * d->H * part_row * sizeof(float)) : 0;
    pl.off_pA = o; o += d->Bt > 1 ? align_up(maps * N * sizeof(float)) : 0;
    pl.off_pD = o; o += d->Bt > 1 ? align_up(maps * sizeof(float)) : 0;
    pl.off_pb = o; o += align_up(maps * sizeof(float));
    pl.off_step = o; o += pl.step_outside ? align_up(maps * (size_t)d->H * W * sizeof(float)) + 256 : 0;
    pl.off_tail = o; o += align_up((size_t)(W + 16) * (5 * (d->dtype == SCAN2D_BF16 ? 2 : 4) + 1));
    if (av) { pl.off_pAv = o; o += d->Bt > 1 ? align_up(maps * N * sizeof(float)) : 0; }
    if (pl.panels > 1) {
        const size_t one = align_up(maps * N * (size_t)d->H * sizeof(float));
        pl.off_hc = o; o += (size_t)(pl.panels - 1) * one;
        pl.off_qc = o; o += 2 * one;
    }
    pl.total = o;
    *out = pl;
    return true;
}

}  // namespace

size_t bwd_workspace_bytes(const scan2d_desc* d, bool softplus, bool av) {
    BwdPlan pl;
    return make_plan(d, &pl, softplus, av) ? pl.total : 0;
}

// Everything bwd_launch could refuse, without enqueuing anything: the plan and the grid sizes of its launches.
int bwd_check(const scan2d_desc* d, bool softplus, bool av) {
    BwdPlan pl;
    if (!make_plan(d, &pl, softplus, av)) return SCAN2D_ERR_BAD_SHAPE;
    const long long maps = (long long)d->Bt * d->Dc;
    if (pl.small) return (maps + 3) / 4 > 2147483647LL ? SCAN2D_ERR_BAD_SHAPE : SCAN2D_OK;
    const int MPW = (pl.waves * 64 / pl.LG) / pl.NG;
    const int ck_NG = (d->N + pl.k.ckpt_NW - 1) / pl.k.ckpt_NW;
    const int MPW1 = (pl.ck_waves * 64 / pl.ck_LG) / ck_NG;
    const long long wg1 = (maps + MPW1 - 1) / MPW1, wg2 = ((long long)d->Bt * pl.CG + MPW - 1) / MPW;
    if (wg1 > 2147483647LL || wg2 > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
    const long long chunks = ((long long)d->H * d->W + 1023) / 1024;
    if (pl.step_outside && chunks * maps > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
    return SCAN2D_OK;
}

namespace {
bool saving_plan(const scan2d_desc* d, BwdPlan* pl) {
    if (d->flags != 0u || !make_plan(d, pl)) return false;
    return !pl->small && pl->panels == 1 && pl->nb > 1 && pl->k.train_fwd != nullptr && d->N == pl->k.cf_NG * pl->k.cf_NW;
}
}  // namespace

size_t bwd_saved_bytes(const scan2d_desc* d) {
    BwdPlan pl;
    if (!saving_plan(d, &pl)) return 0;
    return align_up((size_t)d->Bt * d->Dc * pl.nb * d->N * (pl.ck_chunked ? (size_t)pl.LG * pl.K : (size_t)d->W) * sizeof(float));
}

int fwd_saving_launch(const scan2d_desc* d, const void* x, const void* delta, const float* A, const void* Bm, const void* Cm,
                      const float* Dskip, const uint8_t* mask, void* y, float* saved, hipStream_t stream) {
    BwdPlan pl;
    if (!saving_plan(d, &pl)) return SCAN2D_ERR_BAD_SHAPE;
    const long long maps = (long long)d->Bt * d->Dc;
    FwdArgs f;
    f.x = x; f.delta = delta; f.A = A; f.Bm = Bm; f.Cm = Cm; f.Dskip = Dskip; f.mask = mask; f.y = y;
    f.delta_bias = nullptr; f.carry = nullptr;
    f.ck = saved; f.nb = pl.nb; f.ck_chunked = pl.ck_chunked ? 1 : 0;
    f.maps = maps; f.Dc = d->Dc; f.H = d->H; f.W = d->W; f.N = d->N;
    const int slots = pl.k.cf_waves * 64 / pl.k.cf_LG;
    f.NG = pl.k.cf_NG; f.MPW = slots / pl.k.cf_NG; f.panels = 1; f.RPB = pl.k.cf_RPB;
    const long long wgf = (maps + f.MPW - 1) / f.MPW;
    if (wgf > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
    const size_t panel = (size_t)pl.k.cf_LG * pl.k.cf_K;
    const size_t lds = (2 * (size_t)f.MPW * f.RPB * 2 * panel + 2 * (size_t)f.RPB * slots * panel) * sizeof(float);
    if (lds > 160 * 1024) return SCAN2D_ERR_BAD_SHAPE;
    (void)hipGetLastError();
    if (lds > 65536 && !allow_large_lds(reinterpret_cast<const void*>(pl.k.train_fwd), lds)) return SCAN2D_ERR_LAUNCH_FAILED;
    hipLaunchKernelGGL(pl.k.train_fwd, dim3((unsigned)wgf), dim3(pl.k.cf_waves * 64), lds, stream, f);
    return hipGetLastError() == hipSuccess ? SCAN2D_OK : SCAN2D_ERR_LAUNCH_FAILED;
}

bool bwd_describe(const scan2d_desc* d, char* text, size_t text_bytes) {
    BwdPlan pl;
    if (!make_plan(d, &pl)) return false;
    const long long maps = (long long)d->Bt * d->Dc;
    long long wgs;
    if (pl.small) wgs = (maps + 3) / 4;
    else wgs = ((long long)d->Bt * pl.CG + (pl.waves * 64 / pl.LG) / pl.NG - 1) / ((pl.waves * 64 / pl.LG) / pl.NG);
    std::snprintf(text, text_bytes, "%sbwd form=%s LG=%d K=%d NW=%d waves=%d RB=%d GS=%d CG=%d bands=%d panels=%d wgs=%lld lds=%zu workspace=%zu",
                  (d->flags & SCAN2D_FLAG_COLUMNS_FIRST) != 0 ? "columns-first(in-kernel) " : "",
                  pl.small ? "small" : (pl.shared ? "banded-shared" : "banded"), pl.LG, pl.K, pl.NW, pl.waves, pl.RB, pl.GS, pl.CG, pl.nb,
                  pl.panels, wgs, pl.lds_bytes, pl.total);
    return true;
}

bool bwd_gate_in_sweep(const scan2d_desc* d) {
    BwdPlan pl;
    return d->flags == 0u && make_plan(d, &pl, true, false) && pl.shared && pl.panels == 1 && !pl.step_outside &&
           pl.k.main_gate != nullptr;
}

namespace {
// Sum of ddelta_raw over positions and batch items, per channel (softplus step only).
void launch_bias_sums(const scan2d_desc* d, const BwdPlan& pl, const void* ddelta_raw, float* dbias, char* ws, hipStream_t stream) {
    const long long maps = (long long)d->Bt * d->Dc;
    const size_t HW = (size_t)d->H * d->W;
    float* pb = d->Bt > 1 ? reinterpret_cast<float*>(ws + pl.off_pb) : dbias;
    if (d->dtype == SCAN2D_BF16)
        hipLaunchKernelGGL(scan2d_bwd_reduce_bias_kernel<bf16_t>, dim3((unsigned)maps), dim3(256), 0, stream,
                           static_cast<const bf16_t*>(ddelta_raw), pb, HW);
    else
        hipLaunchKernelGGL(scan2d_bwd_reduce_bias_kernel<float>, dim3((unsigned)maps), dim3(256), 0, stream,
                           static_cast<const float*>(ddelta_raw), pb, HW);
    if (d->Bt > 1)
        hipLaunchKernelGGL(scan2d_bwd_reduce_bias_batch_kernel, dim3((d->Dc + 255) / 256), dim3(256), 0, stream,
                           pb, dbias, d->Bt, d->Dc);
}
}  // namespace

int bwd_launch(const scan2d_desc* d, const void* x, const void* delta, const float* delta_bias, bool softplus,
               const float* A, const void* Bm,
               const void* Cm, const float* Dskip, const uint8_t* mask, const void* dy, void* dx,
               void* ddelta, float* ddelta_bias, float* dA, float* dBm, float* dCm, float* dDskip, void* workspace,
               size_t workspace_bytes, hipStream_t stream, const float* A_v, float* dA_v, const float* saved,
               const void* z, const void* y_scan, void* dz) {
    BwdPlan pl;
    if (!make_plan(d, &pl, softplus, A_v != nullptr)) return SCAN2D_ERR_BAD_SHAPE;
    if (z != nullptr) {                                        // the output gate's backward inside the main sweep
        if (!softplus || y_scan == nullptr || dz == nullptr || !pl.shared || pl.panels != 1 || pl.step_outside || pl.k.main_gate == nullptr)
            return SCAN2D_ERR_BAD_SHAPE;
        pl.k.main = pl.k.main_gate;
    }
    if (pl.total > 0 && (workspace == nullptr || workspace_bytes < pl.total)) return SCAN2D_ERR_WORKSPACE_SMALL;
    char* ws = static_cast<char*>(workspace);
    BwdArgs a;
    a.x = x; a.delta = delta; a.A = A; a.Bm = Bm; a.Cm = Cm; a.Dskip = Dskip; a.mask = mask; a.dy = dy;
    a.dx = dx; a.ddelta = ddelta; a.delta_bias = delta_bias;
    a.z = z; a.y_scan = y_scan; a.dz = dz;
    if (pl.step_outside) a.delta = ws + pl.off_step;
    a.tail = pl.small ? nullptr : ws + pl.off_tail;
    a.ck = saved != nullptr ? const_cast<float*>(saved) : reinterpret_cast<float*>(ws + pl.off_ck);
    a.pB = pl.CG > 1 ? reinterpret_cast<float*>(ws + pl.off_pB) : dBm;   // one group: the partial is the result
    a.pC = pl.CG > 1 ? reinterpret_cast<float*>(ws + pl.off_pC) : dCm;
    a.pA = d->Bt > 1 ? reinterpret_cast<float*>(ws + pl.off_pA) : dA;
    a.pD = dDskip == nullptr ? nullptr : (d->Bt > 1 ? reinterpret_cast<float*>(ws + pl.off_pD) : dDskip);
    a.Bt = d->Bt; a.Dc = d->Dc; a.H = d->H; a.W = d->W; a.N = d->N;
    a.NG = pl.NG; a.GS = pl.GS; a.CG = pl.CG; a.nb = pl.nb;
    a.A_v = A_v;
    a.ck_chunked = pl.ck_chunked ? 1 : 0;
    a.part_chunked = pl.part_chunked ? 1 : 0;
    a.pAv = A_v == nullptr ? nullptr : (d->Bt > 1 ? reinterpret_cast<float*>(ws + pl.off_pAv) : dA_v);
    // the sweeps that apply the softplus themselves also add up ddelta_raw per map
    const bool bias_in_sweep = softplus && ddelta_bias != nullptr && pl.shared && !pl.step_outside && !pl.small;
    if (bias_in_sweep) a.pBias = d->Bt > 1 ? reinterpret_cast<float*>(ws + pl.off_pb) : ddelta_bias;

    const long long maps = (long long)d->Bt * d->Dc;
    if (pl.small) {
        const long long wgs = (maps + 3) / 4;
        if (wgs > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
        (void)hipGetLastError();
        hipLaunchKernelGGL(pl.k.main, dim3((unsigned)wgs), dim3(256), 0, stream, a);
        if (pl.CG > 1) {
            const size_t NHW = (size_t)d->N * d->H * d->W;
            const size_t total = (size_t)d->Bt * NHW;
            const unsigned blocks = (unsigned)std::min<size_t>((total + 255) / 256, 16384);
            hipLaunchKernelGGL(scan2d_bwd_reduce_groups_kernel, dim3(blocks), dim3(256), 0, stream,
                               a.pB, a.pC, dBm, dCm, d->Bt, pl.CG, NHW);
        }
        if (d->Bt > 1) {
            const int n = d->Dc * d->N;
            hipLaunchKernelGGL(scan2d_bwd_reduce_batch_kernel, dim3((n + 255) / 256), dim3(256), 0, stream,
                               a.pA, a.pD, dA, dDskip, d->Bt, d->Dc, d->N);
        }
        if (softplus && ddelta_bias != nullptr) launch_bias_sums(d, pl, ddelta, ddelta_bias, ws, stream);
        return hipGetLastError() == hipSuccess ? SCAN2D_OK : SCAN2D_ERR_LAUNCH_FAILED;
    }
    const int slots = pl.waves * 64 / pl.LG;
    const int MPW = slots / pl.NG;
    BwdArgs ac = a;                                            // the checkpoint sweep may hold more states per lane
    ac.NG = (d->N + pl.k.ckpt_NW - 1) / pl.k.ckpt_NW;
    const int MPW1 = (pl.ck_waves * 64 / pl.ck_LG) / ac.NG;
    const long long wg1 = (maps + MPW1 - 1) / MPW1;
    const long long jobs = (long long)d->Bt * pl.CG;
    const long long wg2 = (jobs + MPW - 1) / MPW;
    if (wg1 > 2147483647LL || wg2 > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
    (void)hipGetLastError();
    const size_t HW = (size_t)d->H * d->W;
    if (!pl.fast) {
        const size_t r1 = ((size_t)maps - 1) * HW + (size_t)(d->H - 1) * d->W;
        const size_t r2 = ((size_t)d->Bt * d->N - 1) * HW + (size_t)(d->H - 1) * d->W;
        const size_t r3 = ((size_t)d->Bt - 1) * HW + (size_t)(d->H - 1) * d->W;
        if (d->dtype == SCAN2D_BF16)
            hipLaunchKernelGGL(scan2d_bwd_tail_kernel<bf16_t>, dim3(1), dim3(256), 0, stream, static_cast<const bf16_t*>(x),
                               static_cast<const bf16_t*>(delta), static_cast<const bf16_t*>(dy), static_cast<const bf16_t*>(Bm),
                               static_cast<const bf16_t*>(Cm), mask, reinterpret_cast<bf16_t*>(ws + pl.off_tail), r1, r2, r3, d->W);
        else
            hipLaunchKernelGGL(scan2d_bwd_tail_kernel<float>, dim3(1), dim3(256), 0, stream, static_cast<const float*>(x),
                               static_cast<const float*>(delta), static_cast<const float*>(dy), static_cast<const float*>(Bm),
                               static_cast<const float*>(Cm), mask, reinterpret_cast<float*>(ws + pl.off_tail), r1, r2, r3, d->W);
    }
    if (pl.step_outside) {
        const unsigned chunks = (unsigned)((HW + 1023) / 1024);
        if ((long long)chunks * maps > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
        float* step = reinterpret_cast<float*>(ws + pl.off_step);
        if (d->dtype == SCAN2D_BF16)
            hipLaunchKernelGGL(scan2d_bwd_step_kernel<bf16_t>, dim3((unsigned)(chunks * maps)), dim3(256), 0, stream,
                               static_cast<const bf16_t*>(delta), delta_bias, step, HW, d->Dc, chunks);
        else
            hipLaunchKernelGGL(scan2d_bwd_step_kernel<float>, dim3((unsigned)(chunks * maps)), dim3(256), 0, stream,
                               static_cast<const float*>(delta), delta_bias, step, HW, d->Dc, chunks);
    }
    if (pl.lds_bytes > 65536 && !allow_large_lds(reinterpret_cast<const void*>(pl.k.main), pl.lds_bytes)) return SCAN2D_ERR_LAUNCH_FAILED;
    if (pl.panels > 1) {
        // wide maps: checkpoint sweeps left to right (row-end states handed on), main sweeps right to left (a*q handed on)
        const size_t one = align_up((size_t)maps * d->N * d->H * sizeof(float));
        const int PW = pl.LG * pl.K;
        for (int q = 0; q < pl.panels; ++q) {
            BwdArgs c = ac;
            c.cb = q * PW;
            c.hc_in = q > 0 ? reinterpret_cast<const float*>(ws + pl.off_hc + (size_t)(q - 1) * one) : nullptr;
            c.hc_out = q + 1 < pl.panels ? reinterpret_cast<float*>(ws + pl.off_hc + (size_t)q * one) : nullptr;
            hipLaunchKernelGGL(pl.k.ckpt, dim3((unsigned)wg1), dim3(pl.ck_waves * 64), 0, stream, c);
        }
        for (int q = pl.panels - 1; q >= 0; --q) {
            BwdArgs m = a;
            m.cb = q * PW;
            m.hc_in = q > 0 ? reinterpret_cast<const float*>(ws + pl.off_hc + (size_t)(q - 1) * one) : nullptr;
            m.qc_in = q + 1 < pl.panels ? reinterpret_cast<const float*>(ws + pl.off_qc + (size_t)((q + 1) & 1) * one) : nullptr;
            m.qc_out = q > 0 ? reinterpret_cast<float*>(ws + pl.off_qc + (size_t)(q & 1) * one) : nullptr;
            m.accum = q + 1 < pl.panels ? 1 : 0;
            hipLaunchKernelGGL(pl.k.main, dim3((unsigned)wg2), dim3(pl.waves * 64), pl.lds_bytes, stream, m);
        }
    } else {
        if (saved != nullptr) {
            // the forward pass of the training step has left the checkpoints
        } else if (pl.nb > 1 && pl.k.ckpt_fwd != nullptr && d->N == pl.k.cf_NG * pl.k.cf_NW) {
            // the checkpoint sweep by the shared-producer forward kernel (checkpoint mode): it computes the softplus
            // step itself from the raw projection, with the same function as the step kernel above
            FwdArgs f;
            f.x = x; f.delta = delta; f.A = A; f.Bm = Bm; f.Cm = Cm; f.Dskip = nullptr; f.mask = mask; f.y = nullptr;
            f.delta_bias = delta_bias; f.carry = nullptr;
            f.ck = a.ck; f.nb = pl.nb; f.ck_chunked = pl.ck_chunked ? 1 : 0;
            f.maps = maps; f.Dc = d->Dc; f.H = d->H; f.W = d->W; f.N = d->N;
            f.NG = pl.k.cf_NG; f.MPW = (pl.k.cf_waves * 64 / pl.k.cf_LG) / pl.k.cf_NG; f.panels = 1; f.RPB = pl.k.cf_RPB;
            const long long wgf = (maps + f.MPW - 1) / f.MPW;
            if (wgf > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
            const size_t lds_f = 2 * (size_t)f.MPW * f.RPB * 2 * pl.k.cf_LG * pl.k.cf_K * sizeof(float);   // the per-position buffers only
            hipLaunchKernelGGL(pl.k.ckpt_fwd, dim3((unsigned)wgf), dim3(pl.k.cf_waves * 64), lds_f, stream, f);
        } else if (pl.nb > 1) {
            hipLaunchKernelGGL(pl.k.ckpt, dim3((unsigned)wg1), dim3(pl.ck_waves * 64), 0, stream, ac);
        }
        hipLaunchKernelGGL(pl.k.main, dim3((unsigned)wg2), dim3(pl.waves * 64), pl.lds_bytes, stream, a);
    }
    if (pl.CG > 1 && pl.part_chunked) {
        const size_t rows = (size_t)d->N * d->H;
        const size_t total = (size_t)d->Bt * rows * pl.LG * pl.K;
        const unsigned blocks = (unsigned)std::min<size_t>((total + 255) / 256, 16384);
        hipLaunchKernelGGL(scan2d_bwd_reduce_groups_chunked_kernel, dim3(blocks), dim3(256), 0, stream,
                           a.pB, a.pC, dBm, dCm, d->Bt, pl.CG, rows, d->W, pl.LG, pl.K);
    } else if (pl.CG > 1) {
        const size_t NHW = (size_t)d->N * d->H * d->W;
        const size_t total = (size_t)d->Bt * NHW;
        const unsigned blocks = (unsigned)std::min<size_t>((total + 255) / 256, 16384);
        hipLaunchKernelGGL(scan2d_bwd_reduce_groups_kernel, dim3(blocks), dim3(256), 0, stream,
                           a.pB, a.pC, dBm, dCm, d->Bt, pl.CG, NHW);
    }
    if (d->Bt > 1) {
        const int n = d->Dc * d->N;
        hipLaunchKernelGGL(scan2d_bwd_reduce_batch_kernel, dim3((n + 255) / 256), dim3(256), 0, stream,
                           a.pA, a.pD, dA, dDskip, d->Bt, d->Dc, d->N);
        if (A_v != nullptr)
            hipLaunchKernelGGL(scan2d_bwd_reduce_batch_kernel, dim3((n + 255) / 256), dim3(256), 0, stream,
                               a.pAv, static_cast<const float*>(nullptr), dA_v, static_cast<float*>(nullptr), d->Bt, d->Dc, d->N);
    }
    if (pl.step_outside) {
        float* pb = ddelta_bias == nullptr ? nullptr : (d->Bt > 1 ? reinterpret_cast<float*>(ws + pl.off_pb) : ddelta_bias);
        const float* dstep = reinterpret_cast<const float*>(ws + pl.off_step);
        if (d->dtype == SCAN2D_BF16)
            hipLaunchKernelGGL(scan2d_bwd_chain_kernel<bf16_t>, dim3((unsigned)maps), dim3(256), 0, stream, dstep,
                               static_cast<const bf16_t*>(delta), delta_bias, static_cast<bf16_t*>(ddelta), pb, HW, d->Dc);
        else
            hipLaunchKernelGGL(scan2d_bwd_chain_kernel<float>, dim3((unsigned)maps), dim3(256), 0, stream, dstep,
                               static_cast<const float*>(delta), delta_bias, static_cast<float*>(ddelta), pb, HW, d->Dc);
        if (ddelta_bias != nullptr && d->Bt > 1)
            hipLaunchKernelGGL(scan2d_bwd_reduce_bias_batch_kernel, dim3((d->Dc + 255) / 256), dim3(256), 0, stream,
                               pb, ddelta_bias, d->Bt, d->Dc);
    } else if (bias_in_sweep) {
        if (d->Bt > 1)
            hipLaunchKernelGGL(scan2d_bwd_reduce_bias_batch_kernel, dim3((d->Dc + 255) / 256), dim3(256), 0, stream,
                               a.pBias, ddelta_bias, d->Bt, d->Dc);
    } else if (softplus && ddelta_bias != nullptr) {
        launch_bias_sums(d, pl, ddelta, ddelta_bias, ws, stream);
    }
    return hipGetLastError() == hipSuccess ? SCAN2D_OK : SCAN2D_ERR_LAUNCH_FAILED;
}

}  // namespace scan2d
