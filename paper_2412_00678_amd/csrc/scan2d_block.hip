// The two producers in front of the scan inside a 2DMamba block (Sec. 3.2, Fig. 2; Eq. 3 for the projections):
//   scan2d_block_conv_silu_kernel : x = SiLU(depth-wise correlation of u with a KH x KW filter + bias)
//   scan2d_block_xproj_kernel     : low = Wx . x per position (MFMA), Bm / Cm = rows of low, delta_raw = Wdt . low[:R]
// Both write the storage type the scan kernels read, so nothing passes through an fp32 tensor in HBM.
#include "scan2d_block.hpp"

#include <algorithm>

#include "scan2d_common.hpp"

namespace scan2d {
namespace {

template <typename T>
__device__ __forceinline__ float widen_bits(uint32_t bits) {
    if constexpr (Elem<T>::kBytes == 4) return __uint_as_float(bits);
    else return __uint_as_float(bits << 16);
}

// Two fp32 values to a dword of two bf16 (nearest even): one v_cvt_pk_bf16_f32.
typedef float float2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const float2v v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2v));
}

// ------------------------------------------------------------------------------------ convolution + SiLU
// One thread per 4 consecutive outputs of a row.  Per filter row it reads the KW + 3 inputs its outputs need, element
// by element (any width, any alignment; L1 serves the overlap between neighbours), zero outside the map.
template <typename T>
__global__ __launch_bounds__(256) void scan2d_block_conv_silu_kernel(const T* __restrict__ u, const float* __restrict__ w,
                                                                     const float* __restrict__ bias, T* __restrict__ x,
                                                                     long long maps, int Dc, int H, int W, int KH, int KW, int PH, int PW) {
    const int J4 = (W + 3) / 4;
    const long long total = maps * H * J4;
    const long long id = (long long)blockIdx.x * 256 + threadIdx.x;
    if (id >= total) return;
    const int jq = (int)(id % J4);
    const long long t = id / J4;
    const int i = (int)(t % H);
    const long long map = t / H;
    const int c = (int)(map % Dc);
    const int j0 = jq * 4;
    const T* um = u + (size_t)map * H * W;
    const float* wc = w + (size_t)c * KH * KW;
    const float b = bias != nullptr ? bias[c] : 0.0f;
    float acc[4] = {b, b, b, b};
    for (int p = 0; p < KH; ++p) {
        const int ii = i + p - PH;
        if (ii < 0 || ii >= H) continue;
        const T* row = um + (size_t)ii * W;
        float win[10];                                   // KW + 3 <= 10 inputs
#pragma unroll
        for (int e = 0; e < 10; ++e) {
            const int jj = j0 - PW + e;
            win[e] = (e < KW + 3 && jj >= 0 && jj < W) ? widen_bits<T>(elem_bits(row + jj)) : 0.0f;
        }
#pragma unroll
        for (int q = 0; q < 7; ++q) {
            if (q < KW) {
                const float wv = wc[p * KW + q];
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e] = fmaf(wv, win[e + q], acc[e]);
            }
        }
    }
    T* out = x + (size_t)map * H * W + (size_t)i * W + j0;
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if (j0 + e < W) store_elem(out + e, acc[e] * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-acc[e] * kLog2e)));
}

// Wide maps (W >= 32): one workgroup per tile of 32 rows x 64 columns.  The tile and its halo go to LDS as fp32 through
// aligned vector loads (zero outside the map), the channel's filter goes there too, then every thread forms 4 consecutive
// outputs in each of two rows from LDS.  KHC x KWC: the filter size at compile time (0: any size up to 7 x 7).
constexpr int kConvTH = 32, kConvTW = 64, kConvHalo = 8, kConvCols = kConvTW + 2 * kConvHalo;   // 80 columns per tile row
// LDS row pitch: odd, so that the four rows a wavefront reads (lanes: 16 groups of 4 columns x 4 rows) fall on different banks
constexpr int kConvPitch = kConvCols + 1;
template <typename T, int KHC, int KWC>
__global__ __launch_bounds__(256) void scan2d_block_conv_silu_tile_kernel(const T* __restrict__ u, const float* __restrict__ w,
                                                                          const float* __restrict__ bias, T* __restrict__ x,
                                                                          int Dc, int H, int W, int KHr, int KWr, int PH, int PW,
                                                                          int tiles_w, int tiles_h) {
    constexpr int EB = Elem<T>::kBytes;
    const int KH = KHC > 0 ? KHC : KHr, KW = KWC > 0 ? KWC : KWr;
    __shared__ __align__(16) float tile[(kConvTH + 6) * kConvPitch];
    __shared__ float wts[52];
    const int tid = threadIdx.x;
    const int tw = blockIdx.x % tiles_w;
    const int th = (blockIdx.x / tiles_w) % tiles_h;
    const long long map = blockIdx.x / (tiles_w * tiles_h);
    const int c = (int)(map % Dc);
    const int i0 = th * kConvTH, j0 = tw * kConvTW;
    const T* um = u + (size_t)map * H * W;
    const int rows = min(kConvTH, H - i0) + KH - 1;
    const bool vec_ok = (W % 4) == 0;                     // rows and maps then start on vector boundaries
    if (tid < KH * KW) wts[tid] = w[(size_t)c * KH * KW + tid];
    if (tid == 63) wts[49] = bias != nullptr ? bias[c] : 0.0f;
    for (int idx = tid; idx < rows * (kConvCols / 4); idx += 256) {
        const int r = idx / (kConvCols / 4), q = idx % (kConvCols / 4);
        const int ii = i0 + r - PH, jj = j0 - kConvHalo + 4 * q;
        float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (ii >= 0 && ii < H && jj + 3 >= 0 && jj < W) {
            const T* src = um + (size_t)ii * W + jj;
            if (vec_ok && jj >= 0 && jj + 3 < W) {
                if constexpr (EB == 2) {
                    const uint2 t = *reinterpret_cast<const uint2*>(src);
                    v = make_float4(__uint_as_float(t.x << 16), __uint_as_float(t.x & 0xffff0000u), __uint_as_float(t.y << 16),
                                    __uint_as_float(t.y & 0xffff0000u));
                } else {
                    v = *reinterpret_cast<const float4*>(src);
                }
            } else {
                if (jj >= 0 && jj < W) v.x = widen_bits<T>(elem_bits(src));
                if (jj + 1 >= 0 && jj + 1 < W) v.y = widen_bits<T>(elem_bits(src + 1));
                if (jj + 2 >= 0 && jj + 2 < W) v.z = widen_bits<T>(elem_bits(src + 2));
                if (jj + 3 >= 0 && jj + 3 < W) v.w = widen_bits<T>(elem_bits(src + 3));
            }
        }
        float* dst = tile + r * kConvPitch + 4 * q;
        dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    }
    __syncthreads();
    const int jq = tid % 16, j = j0 + 4 * jq;
    if (j >= W) return;
    const float b = wts[49];
    constexpr int KHM = KHC > 0 ? KHC : 7, KWM = KWC > 0 ? KWC : 7;
    float wreg[KHC > 0 ? KHC * KWC : 1];                  // the filter in registers when its size is known
    if constexpr (KHC > 0) {
#pragma unroll
        for (int k = 0; k < KHC * KWC; ++k) wreg[k] = wts[k];
    }
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int r = tid / 16 + 16 * half;               // output row inside the tile
        const int i = i0 + r;
        if (i >= H) continue;
        float acc[4] = {b, b, b, b};
#pragma unroll
        for (int pp = 0; pp < KHM; ++pp) {
            if (pp < KH) {
                const float* row = tile + (r + pp) * kConvPitch + kConvHalo + 4 * jq - PW;
                float win[KWM + 3];
#pragma unroll
                for (int e = 0; e < KWM + 3; ++e) win[e] = e < KW + 3 ? row[e] : 0.0f;
#pragma unroll
                for (int q = 0; q < KWM; ++q) {
                    if (q < KW) {
                        const float wv = KHC > 0 ? wreg[KHC > 0 ? pp * KWC + q : 0] : wts[pp * KW + q];
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[e] = fmaf(wv, win[e + q], acc[e]);
                    }
                }
            }
        }
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = acc[e] * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-acc[e] * kLog2e));   // SiLU: v_exp, v_rcp
        T* out = x + (size_t)map * H * W + (size_t)i * W + j;
        if (vec_ok && j + 3 < W) {
            if constexpr (EB == 2) {
                uint2 t;
                t.x = pack_bf16x2(o[0], o[1]);
                t.y = pack_bf16x2(o[2], o[3]);
                *reinterpret_cast<uint2*>(out) = t;
            } else {
                *reinterpret_cast<float4*>(out) = make_float4(o[0], o[1], o[2], o[3]);
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (j + e < W) store_elem(out + e, o[e]);
        }
    }
}

// ------------------------------------------------------------------------------------ projections
// One workgroup of 4 wavefronts per tile of 64 positions of one batch item.
//   1. a chunk of the tile of x (up to kChunk channels x 64 positions) goes to LDS with vector loads and stores (rows
//      padded so that the four k-groups of a wavefront read different banks);
//   2. low[m][pos] = sum_c Wx[m][c] * x[c][pos] with MFMA 16x16 tiles: a wavefront owns 16 positions and walks over
//      the row blocks of Wx three at a time, over all chunks (bf16 storage: v_mfma_f32_16x16x16_bf16, fp32 storage:
//      v_mfma_f32_16x16x4_f32; fp32 accumulation either way).  The contraction index of an MFMA lane is 4 consecutive
//      channels at one position: x is channel-major in memory, hence the trip through LDS.  The Wx fragments of the
//      next step are requested before the current step's MFMAs.  Rows R..R+2N-1 are rounded and stored as Bm / Cm;
//      rows 0..R-1 stay in LDS as fp32;
//   3. delta_raw[c][pos] = sum_r Wdt[c][r] * low[r][pos] with v_mfma_f32_16x16x4_f32 (fp32 in, fp32 out: low is not
//      rounded), 16 channels x 16 positions per tile; the results are rounded, staged in the LDS rows that held x and
//      written out as whole 128- or 256-byte rows.
constexpr int kTile = 64;
template <typename T> struct XprojTile;
template <> struct XprojTile<bf16_t> { static constexpr int kStep = 16, kPitch = 68, kChunk = 256; };   // 136 B rows: 4 rows apart = 32 B mod 128
template <> struct XprojTile<float>  { static constexpr int kStep = 4,  kPitch = 80, kChunk = 128; };   // 320 B rows: 1 row apart = 64 B mod 128

typedef short short4v __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));

struct XprojArgs {
    const void* x; const void* Wx; const float* Wdt;
    void* delta_raw; void* Bm; void* Cm;
    int Dc, N, R, tiles, Bt;     // tiles per batch item, batch items
    int wdt_lds;                 // Wdt fits the LDS (rows of R rounded up to 4, plus 1, floats)
    long long P;                 // positions per map
};

// KSTM: upper bound of ceil(R / 4), sizes the register arrays of the last product (2: R <= 8, 4: R <= 16, 16: R <= 64)
// ALIGNED: H*W and Dc are multiples of 4, so every group of 4 positions / 4 channels is one aligned vector that lies
// inside its row or outside it as a whole.  Those instantiations contain no element-wise path and no load in a branch
// (addresses are clamped, values selected): with the two paths side by side the compiler's wait counts serialise the
// loads, which cost a factor of three.
template <typename T, int KSTM, bool ALIGNED>
__global__ __launch_bounds__(256) void scan2d_block_xproj_kernel(const XprojArgs p) {
    constexpr int KS = XprojTile<T>::kStep, PT = XprojTile<T>::kPitch, KC = XprojTile<T>::kChunk;
    constexpr int EB = Elem<T>::kBytes;
    using Raw = std::conditional_t<EB == 2, uint16_t, uint32_t>;
    using Frag = std::conditional_t<EB == 2, short4v, float>;
    extern __shared__ __align__(16) unsigned char smem[];
    const int Dc = p.Dc, N = p.N, R = p.R, M = R + 2 * N;
    const int Rp = (R + 3) & ~3;
    Raw* xs = reinterpret_cast<Raw*>(smem);                                    // [KC][PT]
    float* dtl = reinterpret_cast<float*>(smem + (size_t)KC * PT * EB);        // [Rp][kTile]
    float* wdtL = dtl + Rp * kTile;                                            // [Dc][Rp + 1] when p.wdt_lds
    const int tid = threadIdx.x;
    const long long P = p.P;
    const int l = tid & 63, wv = tid >> 6, g = l >> 4, n = l & 15;
    const int ncol = wv * 16 + n;                         // position inside the tile
    const T* Wx = static_cast<const T*>(p.Wx);
    const int MB = (M + 15) / 16;

    auto load_a = [&](int mblock, int k) -> Frag {        // the Wx fragment of row block `mblock` for channels k..
        const int mrow = min(mblock * 16 + n, M - 1);     // rows past M are computed and dropped
        if constexpr (EB == 2) {
            const int kk = k + 4 * g;
            short4v af;
            if constexpr (ALIGNED) {
                const uint2 t = *reinterpret_cast<const uint2*>(Wx + (size_t)mrow * Dc + min(kk, Dc - 4));
                const uint32_t lo = kk < Dc ? t.x : 0u, hi = kk < Dc ? t.y : 0u;
                af.x = (short)(lo & 0xffffu); af.y = (short)(lo >> 16); af.z = (short)(hi & 0xffffu); af.w = (short)(hi >> 16);
            } else {
                const T* src = Wx + (size_t)mrow * Dc + kk;
                af.x = kk     < Dc ? (short)elem_bits(src)     : (short)0;
                af.y = kk + 1 < Dc ? (short)elem_bits(src + 1) : (short)0;
                af.z = kk + 2 < Dc ? (short)elem_bits(src + 2) : (short)0;
                af.w = kk + 3 < Dc ? (short)elem_bits(src + 3) : (short)0;
            }
            return af;
        } else {
            const int kk = k + g;
            const float v = __uint_as_float(elem_bits(Wx + (size_t)mrow * Dc + min(kk, Dc - 1)));
            return kk < Dc ? v : 0.0f;
        }
    };

    // The workgroups are persistent: each walks over tiles blockIdx.x, blockIdx.x + gridDim.x, ...  With at most 48
    // rows of Wx and one chunk of channels (the usual block: N = 16, R <= 16, Dc <= 256 in bf16) the Wx fragments
    // are loaded once per workgroup and stay in registers for all its tiles.
    constexpr int NKS = KC / KS;                                               // MFMA steps per chunk
    Frag afr[NKS][3];
    const bool hoist = MB <= 3 && Dc <= KC;
    auto load_frags = [&](int m0, int kc0, int kn) {
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
            for (int mb = 0; mb < 3; ++mb)
                afr[ks][mb] = load_a(min(m0 + mb, MB - 1), kc0 + ks * KS);    // zero past Dc
    };
    if (hoist) {
        // Wx goes through LDS once (coalesced rows; the fragments gather 16 rows per load, which the L1 serves badly)
        constexpr int WP = KC + 8;                        // row pitch in elements; 48 rows fit the region of the x tile
        if constexpr (ALIGNED) {                          // Dc is a multiple of 4: vectors of 4 elements, all requested at once
            using Vec = std::conditional_t<EB == 2, uint2, uint4>;
            constexpr int NV = 48 * KC / 4 / 256;
            const int nvec = M * Dc / 4;
            Vec wv4[NV];
#pragma unroll
            for (int it = 0; it < NV; ++it) wv4[it] = *reinterpret_cast<const Vec*>(Wx + 4 * (size_t)min(tid + it * 256, nvec - 1));
#pragma unroll
            for (int it = 0; it < NV; ++it) {
                const int e = 4 * (tid + it * 256);
                if (e < M * Dc) *reinterpret_cast<Vec*>(xs + (e / Dc) * WP + e % Dc) = wv4[it];
            }
        } else {
            for (int idx = tid; idx < M * Dc; idx += 256) xs[(idx / Dc) * WP + idx % Dc] = (Raw)elem_bits(Wx + idx);
        }
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
            for (int mb = 0; mb < 3; ++mb) {
                const Raw* row = xs + (size_t)min(mb * 16 + n, M - 1) * WP;
                if constexpr (EB == 2) {
                    const int kk = ks * KS + 4 * g;
                    short4v af;
                    af.x = kk     < Dc ? (short)row[kk]     : (short)0;
                    af.y = kk + 1 < Dc ? (short)row[kk + 1] : (short)0;
                    af.z = kk + 2 < Dc ? (short)row[kk + 2] : (short)0;
                    af.w = kk + 3 < Dc ? (short)row[kk + 3] : (short)0;
                    afr[ks][mb] = af;
                } else {
                    const int kk = ks * KS + g;
                    afr[ks][mb] = kk < Dc ? __uint_as_float(row[kk]) : 0.0f;
                }
            }
        __syncthreads();
    }
    if (p.wdt_lds) {
        // [ceil16(Dc)][Rp + 1], zero where the channel or the low-rank index does not exist: the fragments of the last
        // product then need neither clamping nor a select
        const int RW = Rp + 1, nw = ((Dc + 15) & ~15) * RW;
        for (int base = 0; base < nw; base += 8 * 256) {
            float wv8[8];
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int idx = min(base + it * 256 + tid, nw - 1);
                const int c = idx / RW, r = idx - c * RW;
                wv8[it] = p.Wdt[(size_t)min(c, Dc - 1) * R + min(r, R - 1)];
                if (c >= Dc || r >= R) wv8[it] = 0.0f;
            }
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int idx = base + it * 256 + tid;
                if (idx < nw) wdtL[idx] = wv8[it];
            }
        }
        // visible after the barriers of the first tile
    }
    const long long total_tiles = (long long)p.tiles * p.Bt;
    // The chunk of x of a tile: every load of the thread is requested before the first is used.
    constexpr int NLD = KC * (kTile / 4) / 256;                                // vectors per thread
    using Vec = std::conditional_t<EB == 2, uint2, uint4>;
    Vec xv[NLD];
    auto issue_x = [&](long long tile, int kc0) {
        const T* xb = static_cast<const T*>(p.x) + (size_t)(tile / p.tiles) * Dc * P;
        const long long p0 = (tile % p.tiles) * kTile;
#pragma unroll
        for (int it = 0; it < NLD; ++it) {
            const int idx = tid + it * 256;
            const int cr = idx / (kTile / 4), q = idx % (kTile / 4);
            const int c = kc0 + cr;
            const long long pos = p0 + 4 * q;
            Vec v{};
            if constexpr (ALIGNED) {
                const Vec t = *reinterpret_cast<const Vec*>(xb + (size_t)min(c, Dc - 1) * P + min(pos, P - 4));
                if (c < Dc && pos < P) v = t;
            } else if (c < Dc) {
                const T* src = xb + (size_t)c * P + pos;
                Raw e[4] = {0, 0, 0, 0};
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    if (pos + t < P) e[t] = (Raw)elem_bits(src + t);
                if constexpr (EB == 2) { v.x = (uint32_t)e[0] | ((uint32_t)e[1] << 16); v.y = (uint32_t)e[2] | ((uint32_t)e[3] << 16); }
                else { v.x = e[0]; v.y = e[1]; v.z = e[2]; v.w = e[3]; }
            }
            xv[it] = v;
        }
    };
    // one row group and one chunk per tile (the hoisted case): the next tile's x is requested before this tile's
    // products and is in flight while they run
    if (hoist && blockIdx.x < total_tiles) issue_x(blockIdx.x, 0);
  for (long long tile = blockIdx.x; tile < total_tiles; tile += gridDim.x) {
    const int b = (int)(tile / p.tiles);
    const long long p0 = (tile % p.tiles) * kTile;
    for (int m0 = 0; m0 < MB; m0 += 3) {
        float4v acc[3];
#pragma unroll
        for (int mb = 0; mb < 3; ++mb) acc[mb] = float4v{0.0f, 0.0f, 0.0f, 0.0f};
        for (int kc0 = 0; kc0 < Dc; kc0 += KC) {
            const int kn = min(KC, (Dc - kc0 + KS - 1) / KS * KS);             // rows of this chunk, zero-filled past Dc
            if (!hoist) issue_x(tile, kc0);
            if (!hoist) load_frags(m0, kc0, kn);
            __syncthreads();                                                   // the previous chunk (or tile) has been consumed
#pragma unroll
            for (int it = 0; it < NLD; ++it) {
                const int idx = tid + it * 256;
                const int cr = idx / (kTile / 4), q = idx % (kTile / 4);
                *reinterpret_cast<Vec*>(xs + (size_t)cr * PT + 4 * q) = xv[it];   // rows past the chunk's end hold zeros
            }
            if (hoist && tile + gridDim.x < total_tiles) issue_x(tile + gridDim.x, 0);
            __syncthreads();
            // ---- 2. low += Wx[:, chunk] . x[chunk]
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {            // every step and every row block runs: no branch around an MFMA
                const int k0 = ks * KS;
                if constexpr (EB == 2) {
                    short4v bf;
                    const Raw* col = xs + (size_t)(k0 + 4 * g) * PT + ncol;
                    bf.x = (short)col[0]; bf.y = (short)col[PT]; bf.z = (short)col[2 * PT]; bf.w = (short)col[3 * PT];
#pragma unroll
                    for (int mb = 0; mb < 3; ++mb) acc[mb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(afr[ks][mb], bf, acc[mb], 0, 0, 0);
                } else {
                    const float bv = __uint_as_float(xs[(size_t)(k0 + g) * PT + ncol]);
#pragma unroll
                    for (int mb = 0; mb < 3; ++mb) acc[mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(afr[ks][mb], bv, acc[mb], 0, 0, 0);
                }
            }
        }
        const long long pos = p0 + ncol;
#pragma unroll
        for (int mb = 0; mb < 3; ++mb) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int m = (m0 + mb) * 16 + 4 * g + i;  // row of this accumulator element
                const float v = acc[mb][i];
                if (m < R) {
                    dtl[m * kTile + ncol] = v;
                } else if (m < M && pos < P) {
                    T* dst = m < R + N ? static_cast<T*>(p.Bm) + ((size_t)b * N + (m - R)) * P
                                       : static_cast<T*>(p.Cm) + ((size_t)b * N + (m - R - N)) * P;
                    store_elem(dst + pos, v);
                }
            }
        }
    }
    if (tid < (Rp - R) * kTile) dtl[R * kTile + tid] = 0.0f;                  // at most 3 padding rows of 64
    __syncthreads();

    // ---- 3. delta_raw = Wdt . low[:R], kChunk channels at a time
    T* db = static_cast<T*>(p.delta_raw) + (size_t)b * Dc * P;
    const int KST = Rp / 4;                               // MFMA steps over the low-rank index (at most KSTM)
    float bfrag[KSTM];
#pragma unroll
    for (int kk = 0; kk < KSTM; ++kk) bfrag[kk] = kk < KST ? dtl[(4 * kk + g) * kTile + ncol] : 0.0f;
    for (int cc0 = 0; cc0 < Dc; cc0 += KC) {
        const int cn = min(KC, Dc - cc0);
        constexpr int G = 4;                              // row blocks whose weights are in flight together
        const int nblk = (cn + 15) / 16;
        auto load_w = [&](int mbc, float* af) {
            const int c = cc0 + mbc * 16 + n;
            if (p.wdt_lds) {
                const float* wr = wdtL + (size_t)min(c, ((Dc + 15) & ~15) - 1) * (Rp + 1) + g;
#pragma unroll
                for (int kk = 0; kk < KSTM; ++kk) af[kk] = kk < KST ? wr[4 * kk] : 0.0f;
            } else {
                const float* wr = p.Wdt + (size_t)min(c, Dc - 1) * R;
#pragma unroll
                for (int kk = 0; kk < KSTM; ++kk) {       // unconditional loads from clamped addresses: no load sits in a branch
                    const float v = wr[min(4 * kk + g, R - 1)];
                    af[kk] = (4 * kk + g < R && c < Dc && mbc < nblk) ? v : 0.0f;
                }
            }
        };
        float afn[G][KSTM];
#pragma unroll
        for (int u = 0; u < G; ++u) load_w(u, afn[u]);
        for (int mg = 0; mg < nblk; mg += G) {
            float af[G][KSTM];
#pragma unroll
            for (int u = 0; u < G; ++u)
#pragma unroll
                for (int kk = 0; kk < KSTM; ++kk) af[u][kk] = afn[u][kk];
            if (mg + G < nblk) {
#pragma unroll
                for (int u = 0; u < G; ++u) load_w(mg + G + u, afn[u]);
            }
#pragma unroll
            for (int u = 0; u < G; ++u) {
                const int mbc = mg + u;
                float4v acc = float4v{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int kk = 0; kk < KSTM; ++kk) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(af[u][kk], bfrag[kk], acc, 0, 0, 0);
                if (mbc < nblk) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if constexpr (EB == 2) xs[(size_t)(mbc * 16 + 4 * g + i) * PT + ncol] = (Raw)(pack_bf16x2(acc[i], 0.0f) & 0xffffu);
                        else xs[(size_t)(mbc * 16 + 4 * g + i) * PT + ncol] = __float_as_uint(acc[i]);
                    }
                }
            }
        }
        __syncthreads();
        for (int idx = tid; idx < cn * (kTile / 4); idx += 256) {
            const int cr = idx / (kTile / 4), q = idx % (kTile / 4);
            const long long pos = p0 + 4 * q;
            T* dst = db + (size_t)(cc0 + cr) * P + pos;
            const Raw* src = xs + (size_t)cr * PT + 4 * q;
            if constexpr (ALIGNED) {
                using Vec = std::conditional_t<EB == 2, uint2, uint4>;
                if (pos < P) *reinterpret_cast<Vec*>(dst) = *reinterpret_cast<const Vec*>(src);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (pos + e < P) reinterpret_cast<Raw*>(dst)[e] = src[e];
            }
        }
        __syncthreads();
    }
  }
}

// The common case as a kernel of its own, written for a low instruction count (the general kernel above spends most of
// its time on guards and address arithmetic): H*W a multiple of 64, Dc a multiple of 16 and at most one chunk, at most 48
// rows of Wx, Wdt in LDS.  Nothing in the tile loop is guarded.  All rows of `low` go to an fp32 LDS tile; Bm / Cm are
// rounded and written from there as whole rows, like delta_raw.
template <typename T, int KSTM>
__global__ __launch_bounds__(256) void scan2d_block_xproj_fast_kernel(const XprojArgs p) {
    constexpr int KS = XprojTile<T>::kStep, PT = XprojTile<T>::kPitch, KC = XprojTile<T>::kChunk;
    constexpr int EB = Elem<T>::kBytes, NKS = KC / KS, NLD = KC * (kTile / 4) / 256, LP = kTile + 4;   // LP: pitch of `low`
    using Raw = std::conditional_t<EB == 2, uint16_t, uint32_t>;
    using Frag = std::conditional_t<EB == 2, short4v, float>;
    using Vec = std::conditional_t<EB == 2, uint2, uint4>;
    extern __shared__ __align__(16) unsigned char smem[];
    const int Dc = p.Dc, N = p.N, R = p.R, M = R + 2 * N;
    constexpr int RW = 4 * KSTM + 1;                                           // pitch of Wdt in LDS, zero past R
    Raw* xs = reinterpret_cast<Raw*>(smem);                                    // [KC][PT]
    float* low = reinterpret_cast<float*>(smem + (size_t)KC * PT * EB);        // [48][LP]
    float* wdtL = low + 48 * LP;                                               // [Dc][RW]
    const int tid = threadIdx.x;
    const long long P = p.P;
    const int l = tid & 63, wv = tid >> 6, g = l >> 4, n = l & 15;
    const int ncol = wv * 16 + n;
    const T* Wx = static_cast<const T*>(p.Wx);
    const int n16 = Dc / 16;                                                   // 16-channel row blocks

    // ---- once per workgroup: Wx through LDS into fragment registers, Wdt into LDS
    Frag afr[NKS][3];
    {
        constexpr int WP = KC + 8, NV = 48 * KC / 4 / 256;
        const int nvec = M * Dc / 4;
        Vec wv4[NV];
#pragma unroll
        for (int it = 0; it < NV; ++it) wv4[it] = *reinterpret_cast<const Vec*>(Wx + 4 * (size_t)min(tid + it * 256, nvec - 1));
#pragma unroll
        for (int it = 0; it < NV; ++it) {
            const int e = 4 * (tid + it * 256);
            if (e < M * Dc) *reinterpret_cast<Vec*>(xs + (e / Dc) * WP + e % Dc) = wv4[it];
        }
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
            for (int mb = 0; mb < 3; ++mb) {
                const Raw* row = xs + (size_t)min(mb * 16 + n, M - 1) * WP;
                if constexpr (EB == 2) {
                    const int kk = ks * KS + 4 * g;
                    const uint2 t = *reinterpret_cast<const uint2*>(row + min(kk, Dc - 4));
                    const uint32_t lo = kk < Dc ? t.x : 0u, hi = kk < Dc ? t.y : 0u;
                    short4v af;
                    af.x = (short)(lo & 0xffffu); af.y = (short)(lo >> 16); af.z = (short)(hi & 0xffffu); af.w = (short)(hi >> 16);
                    afr[ks][mb] = af;
                } else {
                    const int kk = ks * KS + g;
                    afr[ks][mb] = kk < Dc ? __uint_as_float(row[min(kk, Dc - 1)]) : 0.0f;
                }
            }
        const int nw = Dc * RW;
        for (int base = 0; base < nw; base += 8 * 256) {
            float wv8[8];
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int idx = min(base + it * 256 + tid, nw - 1);
                const int c = idx / RW, r = idx - c * RW;
                wv8[it] = p.Wdt[(size_t)c * R + min(r, R - 1)];
                if (r >= R) wv8[it] = 0.0f;
            }
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int idx = base + it * 256 + tid;
                if (idx < nw) wdtL[idx] = wv8[it];
            }
        }
        __syncthreads();
    }

    const long long total_tiles = (long long)p.tiles * p.Bt;
    const int cr0 = tid >> 4, q = tid & 15;
    const size_t lane_off = (size_t)cr0 * P + 4 * q;                           // this thread's first vector inside a tile
    const size_t row_step = (size_t)16 * P;                                    // 16 channels further
    Vec xv[NLD];
    auto issue_x = [&](long long tile) {
        const T* src = static_cast<const T*>(p.x) + (size_t)(tile / p.tiles) * Dc * P + (size_t)(tile % p.tiles) * kTile + lane_off;
#pragma unroll
        for (int it = 0; it < NLD; ++it) {
            const Vec t = *reinterpret_cast<const Vec*>(src + (size_t)min(it, n16 - 1) * row_step);
            xv[it] = it < n16 ? t : Vec{};
        }
    };
    if (blockIdx.x < total_tiles) issue_x(blockIdx.x);
    Raw* const xs_mine = xs + (size_t)cr0 * PT + 4 * q;
    const Raw* const xs_col = xs + (size_t)(EB == 2 ? 4 * g : g) * PT + ncol;
    float* const low_mine = low + (4 * g) * LP + ncol;
    const float* const w_mine = wdtL + (size_t)n * RW + g;
    Raw* const stage_mine = xs + (size_t)(4 * g) * PT + ncol;

    for (long long tile = blockIdx.x; tile < total_tiles; tile += gridDim.x) {
        const int b = (int)(tile / p.tiles);
        const long long p0 = (tile % p.tiles) * kTile;
#pragma unroll
        for (int it = 0; it < NLD; ++it) *reinterpret_cast<Vec*>(xs_mine + (size_t)it * 16 * PT) = xv[it];
        if (tile + gridDim.x < total_tiles) issue_x(tile + gridDim.x);          // in flight during this tile's products
        __syncthreads();
        // ---- low = Wx . x
        float4v acc[3];
#pragma unroll
        for (int mb = 0; mb < 3; ++mb) acc[mb] = float4v{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            if constexpr (EB == 2) {
                const Raw* col = xs_col + (size_t)ks * KS * PT;
                short4v bf;
                bf.x = (short)col[0]; bf.y = (short)col[PT]; bf.z = (short)col[2 * PT]; bf.w = (short)col[3 * PT];
#pragma unroll
                for (int mb = 0; mb < 3; ++mb) acc[mb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(afr[ks][mb], bf, acc[mb], 0, 0, 0);
            } else {
                const float bv = __uint_as_float(xs_col[(size_t)ks * KS * PT]);
#pragma unroll
                for (int mb = 0; mb < 3; ++mb) acc[mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(afr[ks][mb], bv, acc[mb], 0, 0, 0);
            }
        }
#pragma unroll
        for (int mb = 0; mb < 3; ++mb)
#pragma unroll
            for (int i = 0; i < 4; ++i) low_mine[(mb * 16 + i) * LP] = acc[mb][i];
        __syncthreads();
        // ---- delta_raw = Wdt . low[:R], staged in the rows that held x
        float bfrag[KSTM];
#pragma unroll
        for (int kk = 0; kk < KSTM; ++kk) {
            const float v = low[(4 * kk + g) * LP + ncol];
            bfrag[kk] = 4 * kk + g < R ? v : 0.0f;
        }
        for (int mbc = 0; mbc < n16; ++mbc) {
            const float* wr = w_mine + (size_t)mbc * 16 * RW;
            float4v d4 = float4v{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int kk = 0; kk < KSTM; ++kk) d4 = __builtin_amdgcn_mfma_f32_16x16x4f32(wr[4 * kk], bfrag[kk], d4, 0, 0, 0);
            Raw* st = stage_mine + (size_t)mbc * 16 * PT;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if constexpr (EB == 2) st[i * PT] = (Raw)(pack_bf16x2(d4[i], 0.0f) & 0xffffu);
                else st[i * PT] = __float_as_uint(d4[i]);
            }
        }
        __syncthreads();
        // ---- whole rows out: delta_raw from the staging rows, Bm / Cm from `low`
        T* db = static_cast<T*>(p.delta_raw) + (size_t)b * Dc * P + p0 + lane_off;
        for (int it = 0; it < n16; ++it)
            *reinterpret_cast<Vec*>(db + (size_t)it * row_step) = *reinterpret_cast<const Vec*>(xs_mine + (size_t)it * 16 * PT);
        for (int idx = tid; idx < 2 * N * (kTile / 4); idx += 256) {
            const int row = idx >> 4, qq = idx & 15;                           // row of Bm (row < N) or Cm
            const float4 v = *reinterpret_cast<const float4*>(low + (R + row) * LP + 4 * qq);
            T* dst = (row < N ? static_cast<T*>(p.Bm) + ((size_t)b * N + row) * P : static_cast<T*>(p.Cm) + ((size_t)b * N + row - N) * P) + p0 + 4 * qq;
            if constexpr (EB == 2) {
                uint2 o;
                o.x = pack_bf16x2(v.x, v.y); o.y = pack_bf16x2(v.z, v.w);
                *reinterpret_cast<uint2*>(dst) = o;
            } else {
                *reinterpret_cast<float4*>(dst) = v;
            }
        }
        __syncthreads();
    }
}

// More channels than one chunk (Dc up to 512, R <= 16, otherwise the conditions of the kernel above): one workgroup per
// compute unit keeps all of Wx in LDS for its whole life (rows padded so that the 16 lanes of a k-group read different
// banks with one wide load each) and the Wdt fragments in registers; x goes through LDS chunk by chunk, the next chunk
// (or the next tile's first) in flight during the products.  The contraction runs over the channels of a 16-channel
// group in the order (lane's k-group, step) instead of (step, k-group): the same permutation on both operands, so each
// lane takes its four Wx values of a group with one 128-bit read (fp32 storage).
constexpr int kWideBlocks = 32;                                               // 16-channel blocks: Dc <= 512
template <typename T> struct XprojWide;
template <> struct XprojWide<bf16_t> { static constexpr int kPitch = 68, kPad = 8; };
template <> struct XprojWide<float>  { static constexpr int kPitch = 68, kPad = 4; };   // 4 rows apart = 64 B mod 256
template <typename T, int KSTM>
__global__ __launch_bounds__(256) void scan2d_block_xproj_wide_kernel(const XprojArgs p) {
    constexpr int KC = XprojTile<T>::kChunk, PT = XprojWide<T>::kPitch;
    constexpr int EB = Elem<T>::kBytes, NLD = KC * (kTile / 4) / 256, LP = kTile + 4, CB = KC / 16;   // CB: blocks per chunk
    using Raw = std::conditional_t<EB == 2, uint16_t, uint32_t>;
    using Vec = std::conditional_t<EB == 2, uint2, uint4>;
    extern __shared__ __align__(16) unsigned char smem[];
    const int Dc = p.Dc, N = p.N, R = p.R, M = R + 2 * N;
    constexpr int RW = 4 * KSTM + 1;
    const int WP = Dc + XprojWide<T>::kPad;                                    // pitch of a Wx row in LDS
    Raw* wxL = reinterpret_cast<Raw*>(smem);                                   // [48][WP]
    Raw* xs = wxL + (size_t)48 * WP;                                           // [KC][PT]
    float* low = reinterpret_cast<float*>(smem + ((size_t)48 * WP + (size_t)KC * PT) * EB);   // [48][LP]
    const int tid = threadIdx.x;
    const long long P = p.P;
    const int l = tid & 63, wv = tid >> 6, g = l >> 4, n = l & 15;
    const int ncol = wv * 16 + n;
    const T* Wx = static_cast<const T*>(p.Wx);
    const int n16 = Dc / 16, NC = (n16 + CB - 1) / CB;

    // ---- once per workgroup: Wdt through the x region into fragment registers, Wx into LDS
    float wfr[kWideBlocks][KSTM];
    {
        float* wdtL = reinterpret_cast<float*>(xs);                            // [Dc][RW], zero past R
        const int nw = Dc * RW;
        for (int base = 0; base < nw; base += 8 * 256) {
            float wv8[8];
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int idx = min(base + it * 256 + tid, nw - 1);
                const int c = idx / RW, r = idx - c * RW;
                wv8[it] = p.Wdt[(size_t)c * R + min(r, R - 1)];
                if (r >= R) wv8[it] = 0.0f;
            }
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int idx = base + it * 256 + tid;
                if (idx < nw) wdtL[idx] = wv8[it];
            }
        }
        const int nvec = M * Dc / 4;
        for (int base = 0; base < nvec; base += 8 * 256) {
            Vec wv4[8];
#pragma unroll
            for (int it = 0; it < 8; ++it) wv4[it] = *reinterpret_cast<const Vec*>(Wx + 4 * (size_t)min(base + it * 256 + tid, nvec - 1));
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int e = 4 * (base + it * 256 + tid);
                if (e < M * Dc) *reinterpret_cast<Vec*>(wxL + (size_t)(e / Dc) * WP + e % Dc) = wv4[it];
            }
        }
        __syncthreads();
#pragma unroll
        for (int mbc = 0; mbc < kWideBlocks; ++mbc)
#pragma unroll
            for (int kk = 0; kk < KSTM; ++kk)
                wfr[mbc][kk] = wdtL[(size_t)(min(mbc, n16 - 1) * 16 + n) * RW + 4 * kk + g];
        __syncthreads();
    }

    const long long total_tiles = (long long)p.tiles * p.Bt;
    const int cr0 = tid >> 4, q = tid & 15;
    const size_t lane_off = (size_t)cr0 * P + 4 * q;
    const size_t row_step = (size_t)16 * P;
    Vec xv[NLD];
    auto issue_x = [&](long long tile, int chunk) {       // rows past Dc: a valid row is read and zeros are kept
        const T* src = static_cast<const T*>(p.x) + (size_t)(tile / p.tiles) * Dc * P + (size_t)(tile % p.tiles) * kTile + lane_off;
        const int nb = n16 - chunk * CB;                   // blocks of this chunk (may exceed CB)
#pragma unroll
        for (int it = 0; it < NLD; ++it) {
            const Vec t = *reinterpret_cast<const Vec*>(src + (size_t)(chunk * CB + min(it, nb - 1)) * row_step);
            xv[it] = it < nb ? t : Vec{};
        }
    };
    if (blockIdx.x < total_tiles) issue_x(blockIdx.x, 0);
    Raw* const xs_mine = xs + (size_t)cr0 * PT + 4 * q;
    const Raw* const xs_col = xs + (size_t)(4 * g) * PT + ncol;
    float* const low_mine = low + (4 * g) * LP + ncol;
    Raw* const stage_mine = xs + (size_t)(4 * g) * PT + ncol;
    const Raw* wrow[3];
#pragma unroll
    for (int mb = 0; mb < 3; ++mb) wrow[mb] = wxL + (size_t)min(mb * 16 + n, M - 1) * WP + 4 * g;

    for (long long tile = blockIdx.x; tile < total_tiles; tile += gridDim.x) {
        const int b = (int)(tile / p.tiles);
        const long long p0 = (tile % p.tiles) * kTile;
        float4v acc[3];
#pragma unroll
        for (int mb = 0; mb < 3; ++mb) acc[mb] = float4v{0.0f, 0.0f, 0.0f, 0.0f};
        // ---- low = Wx . x, chunk by chunk
        for (int chunk = 0; chunk < NC; ++chunk) {
#pragma unroll
            for (int it = 0; it < NLD; ++it) *reinterpret_cast<Vec*>(xs_mine + (size_t)it * 16 * PT) = xv[it];
            if (chunk + 1 < NC) issue_x(tile, chunk + 1);
            else if (tile + gridDim.x < total_tiles) issue_x(tile + gridDim.x, 0);
            __syncthreads();
            const int nb = min(CB, n16 - chunk * CB);      // 16-channel groups of this chunk
            if constexpr (EB == 2) {
                uint2 a_cur[3], a_nxt[3];
                uint16_t b_cur[4], b_nxt[4];
                auto fetch = [&](int kg, uint2* a, uint16_t* bv) {
#pragma unroll
                    for (int mb = 0; mb < 3; ++mb) a[mb] = *reinterpret_cast<const uint2*>(wrow[mb] + chunk * KC + kg * 16);
                    const Raw* col = xs_col + (size_t)kg * 16 * PT;
#pragma unroll
                    for (int i = 0; i < 4; ++i) bv[i] = col[i * PT];
                };
                fetch(0, a_cur, b_cur);
                for (int kg = 0; kg < nb; ++kg) {
                    fetch(min(kg + 1, nb - 1), a_nxt, b_nxt);
                    short4v bf;
                    bf.x = (short)b_cur[0]; bf.y = (short)b_cur[1]; bf.z = (short)b_cur[2]; bf.w = (short)b_cur[3];
#pragma unroll
                    for (int mb = 0; mb < 3; ++mb) {
                        short4v af;
                        af.x = (short)(a_cur[mb].x & 0xffffu); af.y = (short)(a_cur[mb].x >> 16);
                        af.z = (short)(a_cur[mb].y & 0xffffu); af.w = (short)(a_cur[mb].y >> 16);
                        acc[mb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(af, bf, acc[mb], 0, 0, 0);
                    }
#pragma unroll
                    for (int mb = 0; mb < 3; ++mb) a_cur[mb] = a_nxt[mb];
#pragma unroll
                    for (int i = 0; i < 4; ++i) b_cur[i] = b_nxt[i];
                }
            } else {
                float4 a_cur[3], a_nxt[3];
                float b_cur[4], b_nxt[4];
                auto fetch = [&](int kg, float4* a, float* bv) {
#pragma unroll
                    for (int mb = 0; mb < 3; ++mb) a[mb] = *reinterpret_cast<const float4*>(wrow[mb] + chunk * KC + kg * 16);
                    const Raw* col = xs_col + (size_t)kg * 16 * PT;
#pragma unroll
                    for (int i = 0; i < 4; ++i) bv[i] = __uint_as_float(col[i * PT]);
                };
                fetch(0, a_cur, b_cur);
                for (int kg = 0; kg < nb; ++kg) {
                    fetch(min(kg + 1, nb - 1), a_nxt, b_nxt);
#pragma unroll
                    for (int mb = 0; mb < 3; ++mb) {
                        acc[mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a_cur[mb].x, b_cur[0], acc[mb], 0, 0, 0);
                        acc[mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a_cur[mb].y, b_cur[1], acc[mb], 0, 0, 0);
                        acc[mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a_cur[mb].z, b_cur[2], acc[mb], 0, 0, 0);
                        acc[mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a_cur[mb].w, b_cur[3], acc[mb], 0, 0, 0);
                    }
#pragma unroll
                    for (int mb = 0; mb < 3; ++mb) a_cur[mb] = a_nxt[mb];
#pragma unroll
                    for (int i = 0; i < 4; ++i) b_cur[i] = b_nxt[i];
                }
            }
            __syncthreads();                               // the next chunk overwrites the x region
        }
#pragma unroll
        for (int mb = 0; mb < 3; ++mb)
#pragma unroll
            for (int i = 0; i < 4; ++i) low_mine[(mb * 16 + i) * LP] = acc[mb][i];
        __syncthreads();
        // ---- delta_raw = Wdt . low[:R], a chunk of channels at a time through the x region, whole rows out
        float bfrag[KSTM];
#pragma unroll
        for (int kk = 0; kk < KSTM; ++kk) {
            const float v = low[(4 * kk + g) * LP + ncol];
            bfrag[kk] = 4 * kk + g < R ? v : 0.0f;
        }
        T* db = static_cast<T*>(p.delta_raw) + (size_t)b * Dc * P + p0 + lane_off;
#pragma unroll
        for (int mbc = 0; mbc < kWideBlocks; ++mbc) {
            if (mbc < n16) {
                float4v d4 = float4v{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int kk = 0; kk < KSTM; ++kk) d4 = __builtin_amdgcn_mfma_f32_16x16x4f32(wfr[mbc][kk], bfrag[kk], d4, 0, 0, 0);
                Raw* st = stage_mine + (size_t)(mbc % CB) * 16 * PT;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if constexpr (EB == 2) st[i * PT] = (Raw)(pack_bf16x2(d4[i], 0.0f) & 0xffffu);
                    else st[i * PT] = __float_as_uint(d4[i]);
                }
            }
            if ((mbc + 1) % CB == 0 && mbc + 1 - CB < n16) {       // a chunk of rows is staged (uniform)
                const int first = mbc + 1 - CB;
                const int nb = min(CB, n16 - first);
                __syncthreads();
                for (int it = 0; it < nb; ++it)
                    *reinterpret_cast<Vec*>(db + (size_t)(first + it) * row_step) = *reinterpret_cast<const Vec*>(xs_mine + (size_t)it * 16 * PT);
                __syncthreads();
            }
        }
        for (int idx = tid; idx < 2 * N * (kTile / 4); idx += 256) {
            const int row = idx >> 4, qq = idx & 15;
            const float4 v = *reinterpret_cast<const float4*>(low + (R + row) * LP + 4 * qq);
            T* dst = (row < N ? static_cast<T*>(p.Bm) + ((size_t)b * N + row) * P : static_cast<T*>(p.Cm) + ((size_t)b * N + row - N) * P) + p0 + 4 * qq;
            if constexpr (EB == 2) {
                uint2 o;
                o.x = pack_bf16x2(v.x, v.y); o.y = pack_bf16x2(v.z, v.w);
                *reinterpret_cast<uint2*>(dst) = o;
            } else {
                *reinterpret_cast<float4*>(dst) = v;
            }
        }
        __syncthreads();                                   // `low` and the x region are rewritten by the next tile
    }
}

template <typename T>
size_t xproj_wide_lds_bytes(int Dc) {
    return ((size_t)48 * (Dc + XprojWide<T>::kPad) + (size_t)XprojTile<T>::kChunk * XprojWide<T>::kPitch) * Elem<T>::kBytes +
           (size_t)48 * (kTile + 4) * sizeof(float);
}

template <typename T, int KSTM>
size_t xproj_fast_lds_bytes(int Dc) {
    return (size_t)XprojTile<T>::kChunk * XprojTile<T>::kPitch * Elem<T>::kBytes + (size_t)48 * (kTile + 4) * sizeof(float) +
           (size_t)Dc * (4 * KSTM + 1) * sizeof(float);
}

template <typename T>
size_t xproj_lds_bytes(int R) {
    return (size_t)XprojTile<T>::kChunk * XprojTile<T>::kPitch * Elem<T>::kBytes + (size_t)((R + 3) & ~3) * kTile * sizeof(float);
}
size_t xproj_wdt_bytes(int Dc, int R) { return (size_t)((Dc + 15) & ~15) * (((R + 3) & ~3) + 1) * sizeof(float); }

}  // namespace

bool allow_large_lds(const void* kernel, size_t bytes);   // scan2d_api.hip

int block_conv_silu_launch(const scan2d_desc* d, const scan2d_conv_shape* cs, const void* u, const float* w, const float* bias,
                           void* x, hipStream_t stream) {
    if (cs->KH < 1 || cs->KH > 7 || cs->KW < 1 || cs->KW > 7 || cs->PH < 0 || cs->PH >= cs->KH || cs->PW < 0 || cs->PW >= cs->KW)
        return SCAN2D_ERR_BAD_SHAPE;
    const long long maps = (long long)d->Bt * d->Dc;
    (void)hipGetLastError();
    if (d->W >= 32) {                                     // tiles of 16 x 64 outputs staged through LDS
        const int tiles_w = (d->W + kConvTW - 1) / kConvTW, tiles_h = (d->H + kConvTH - 1) / kConvTH;
        const long long wgs = maps * tiles_w * tiles_h;
        if (wgs > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
        const bool k3 = cs->KH == 3 && cs->KW == 3;
        if (d->dtype == SCAN2D_BF16) {
            auto kernel = k3 ? scan2d_block_conv_silu_tile_kernel<bf16_t, 3, 3> : scan2d_block_conv_silu_tile_kernel<bf16_t, 0, 0>;
            hipLaunchKernelGGL(kernel, dim3((unsigned)wgs), dim3(256), 0, stream, static_cast<const bf16_t*>(u), w, bias,
                               static_cast<bf16_t*>(x), d->Dc, d->H, d->W, cs->KH, cs->KW, cs->PH, cs->PW, tiles_w, tiles_h);
        } else {
            auto kernel = k3 ? scan2d_block_conv_silu_tile_kernel<float, 3, 3> : scan2d_block_conv_silu_tile_kernel<float, 0, 0>;
            hipLaunchKernelGGL(kernel, dim3((unsigned)wgs), dim3(256), 0, stream, static_cast<const float*>(u), w, bias,
                               static_cast<float*>(x), d->Dc, d->H, d->W, cs->KH, cs->KW, cs->PH, cs->PW, tiles_w, tiles_h);
        }
        return hipGetLastError() == hipSuccess ? SCAN2D_OK : SCAN2D_ERR_LAUNCH_FAILED;
    }
    const long long total = maps * d->H * ((d->W + 3) / 4);
    const long long blocks = (total + 255) / 256;
    if (blocks > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
    if (d->dtype == SCAN2D_BF16)
        hipLaunchKernelGGL(scan2d_block_conv_silu_kernel<bf16_t>, dim3((unsigned)blocks), dim3(256), 0, stream,
                           static_cast<const bf16_t*>(u), w, bias, static_cast<bf16_t*>(x), maps, d->Dc, d->H, d->W, cs->KH, cs->KW, cs->PH, cs->PW);
    else
        hipLaunchKernelGGL(scan2d_block_conv_silu_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, stream,
                           static_cast<const float*>(u), w, bias, static_cast<float*>(x), maps, d->Dc, d->H, d->W, cs->KH, cs->KW, cs->PH, cs->PW);
    return hipGetLastError() == hipSuccess ? SCAN2D_OK : SCAN2D_ERR_LAUNCH_FAILED;
}

int block_xproj_launch(const scan2d_desc* d, int R, const void* x, const void* Wx, const float* Wdt, void* delta_raw, void* Bm,
                       void* Cm, hipStream_t stream) {
    if (R < 1 || R > 64) return SCAN2D_ERR_BAD_SHAPE;
    const bool bf16 = d->dtype == SCAN2D_BF16;
    {   // the common case: see scan2d_block_xproj_fast_kernel
        const long long P = (long long)d->H * d->W;
        const int kc = bf16 ? XprojTile<bf16_t>::kChunk : XprojTile<float>::kChunk;
        if (P % kTile == 0 && d->Dc % 16 == 0 && d->Dc <= kc && R + 2 * d->N <= 48 && (long long)d->Bt * (P / kTile) <= 2147483647LL) {
            XprojArgs a;
            a.x = x; a.Wx = Wx; a.Wdt = Wdt; a.delta_raw = delta_raw; a.Bm = Bm; a.Cm = Cm;
            a.Dc = d->Dc; a.N = d->N; a.R = R; a.P = P; a.tiles = (int)(P / kTile); a.Bt = d->Bt; a.wdt_lds = 1;
            using Kernel = void (*)(const XprojArgs);
            Kernel kernel;
            size_t lds;
            if (bf16) {
                if (R <= 8) { kernel = scan2d_block_xproj_fast_kernel<bf16_t, 2>; lds = xproj_fast_lds_bytes<bf16_t, 2>(d->Dc); }
                else if (R <= 16) { kernel = scan2d_block_xproj_fast_kernel<bf16_t, 4>; lds = xproj_fast_lds_bytes<bf16_t, 4>(d->Dc); }
                else { kernel = scan2d_block_xproj_fast_kernel<bf16_t, 16>; lds = xproj_fast_lds_bytes<bf16_t, 16>(d->Dc); }
            } else {
                if (R <= 8) { kernel = scan2d_block_xproj_fast_kernel<float, 2>; lds = xproj_fast_lds_bytes<float, 2>(d->Dc); }
                else if (R <= 16) { kernel = scan2d_block_xproj_fast_kernel<float, 4>; lds = xproj_fast_lds_bytes<float, 4>(d->Dc); }
                else { kernel = scan2d_block_xproj_fast_kernel<float, 16>; lds = xproj_fast_lds_bytes<float, 16>(d->Dc); }
            }
            (void)hipGetLastError();
            if (lds > 65536 && !allow_large_lds(reinterpret_cast<const void*>(kernel), lds)) return SCAN2D_ERR_LAUNCH_FAILED;
            const long long grid = std::min<long long>((long long)a.tiles * d->Bt, 2 * 256);
            hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(256), lds, stream, a);
            return hipGetLastError() == hipSuccess ? SCAN2D_OK : SCAN2D_ERR_LAUNCH_FAILED;
        }
    }
    {   // more channels than one chunk: see scan2d_block_xproj_wide_kernel
        const long long P = (long long)d->H * d->W;
        if (P % kTile == 0 && d->Dc % 16 == 0 && d->Dc <= 16 * kWideBlocks && R <= 16 && R + 2 * d->N <= 48 &&
            (long long)d->Bt * (P / kTile) <= 2147483647LL) {
            XprojArgs a;
            a.x = x; a.Wx = Wx; a.Wdt = Wdt; a.delta_raw = delta_raw; a.Bm = Bm; a.Cm = Cm;
            a.Dc = d->Dc; a.N = d->N; a.R = R; a.P = P; a.tiles = (int)(P / kTile); a.Bt = d->Bt; a.wdt_lds = 0;
            using Kernel = void (*)(const XprojArgs);
            Kernel kernel;
            if (bf16) kernel = R <= 8 ? scan2d_block_xproj_wide_kernel<bf16_t, 2> : scan2d_block_xproj_wide_kernel<bf16_t, 4>;
            else kernel = R <= 8 ? scan2d_block_xproj_wide_kernel<float, 2> : scan2d_block_xproj_wide_kernel<float, 4>;
            const size_t lds = bf16 ? xproj_wide_lds_bytes<bf16_t>(d->Dc) : xproj_wide_lds_bytes<float>(d->Dc);
            (void)hipGetLastError();
            if (lds > 65536 && !allow_large_lds(reinterpret_cast<const void*>(kernel), lds)) return SCAN2D_ERR_LAUNCH_FAILED;
            const long long grid = std::min<long long>((long long)a.tiles * d->Bt, 256);   // one workgroup per compute unit (LDS)
            hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(256), lds, stream, a);
            return hipGetLastError() == hipSuccess ? SCAN2D_OK : SCAN2D_ERR_LAUNCH_FAILED;
        }
    }
    size_t lds = bf16 ? xproj_lds_bytes<bf16_t>(R) : xproj_lds_bytes<float>(R);
    const bool wdt_lds = xproj_wdt_bytes(d->Dc, R) <= 40 * 1024;
    if (wdt_lds) lds += xproj_wdt_bytes(d->Dc, R);
    XprojArgs a;
    a.x = x; a.Wx = Wx; a.Wdt = Wdt; a.delta_raw = delta_raw; a.Bm = Bm; a.Cm = Cm;
    a.Dc = d->Dc; a.N = d->N; a.R = R;
    a.P = (long long)d->H * d->W;
    const long long tiles = (a.P + kTile - 1) / kTile;
    if (tiles * d->Bt > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
    a.tiles = (int)tiles; a.Bt = d->Bt; a.wdt_lds = wdt_lds ? 1 : 0;
    (void)hipGetLastError();
    using Kernel = void (*)(const XprojArgs);
    const bool aligned = (a.P % 4) == 0 && (d->Dc % 4) == 0;
    const int kst = R <= 8 ? 2 : (R <= 16 ? 4 : 16);
    Kernel kernel = nullptr;
#define SCAN2D_PICK(T, K)                                                                                          \
    if (kst == K) kernel = aligned ? scan2d_block_xproj_kernel<T, K, true> : scan2d_block_xproj_kernel<T, K, false>;
    if (bf16) { SCAN2D_PICK(bf16_t, 2) SCAN2D_PICK(bf16_t, 4) SCAN2D_PICK(bf16_t, 16) }
    else { SCAN2D_PICK(float, 2) SCAN2D_PICK(float, 4) SCAN2D_PICK(float, 16) }
#undef SCAN2D_PICK
    if (lds > 65536 && !allow_large_lds(reinterpret_cast<const void*>(kernel), lds)) return SCAN2D_ERR_LAUNCH_FAILED;
    const long long grid = std::min<long long>(tiles * d->Bt, 2 * 256);      // two workgroups per compute unit (registers)
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(256), lds, stream, a);
    return hipGetLastError() == hipSuccess ? SCAN2D_OK : SCAN2D_ERR_LAUNCH_FAILED;
}

}  // namespace scan2d
