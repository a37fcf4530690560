// The two producers in front of the scan inside a 2DMamba block (Sec. 3.2, Fig. 2; Eq. 3 for the projections):
//   scan2d_block_conv_silu_kernel : x = SiLU(depth-wise correlation of u with a KH x KW filter + bias)
//   scan2d_block_xproj_kernel     : low = Wx . x per position (MFMA), Bm / Cm = rows of low, delta_raw = Wdt . low[:R]
// Both write the storage type the scan kernels read, so nothing passes through an fp32 tensor in HBM.
#include "scan2d_block.hpp"

#include "scan2d_common.hpp"

namespace scan2d {
namespace {

template <typename T>
__device__ __forceinline__ float widen_bits(uint32_t bits) {
    if constexpr (Elem<T>::kBytes == 4) return __uint_as_float(bits);
    else return __uint_as_float(bits << 16);
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
        if (j0 + e < W) store_elem(out + e, acc[e] / (1.0f + __expf(-acc[e])));
}

// ------------------------------------------------------------------------------------ projections
// One workgroup of 4 wavefronts per tile of 64 positions of one batch item.
//   1. the tile of x, all Dc channels x 64 positions, goes to LDS (rows padded so that the four k-groups of a
//      wavefront read different banks);
//   2. low[m][pos] = sum_c Wx[m][c] * x[c][pos] with MFMA 16x16 tiles: a wavefront owns 16 positions and walks over
//      the row blocks of Wx three at a time (bf16 storage: v_mfma_f32_16x16x16_bf16, fp32 storage:
//      v_mfma_f32_16x16x4_f32; fp32 accumulation either way).  The contraction index of an MFMA lane is 4 consecutive
//      channels at one position: x is channel-major in memory, hence the trip through LDS.  Rows R..R+2N-1 are
//      rounded and stored as Bm / Cm; rows 0..R-1 stay in LDS as fp32;
//   3. delta_raw[c][pos] = sum_r Wdt[c][r] * low[r][pos] in fp32 FMAs (R is 8..64: too thin for an MFMA tile without
//      rounding low to bf16), 4 positions per thread, stored as one vector per thread.
constexpr int kTile = 64;
template <typename T> struct XprojTile;
template <> struct XprojTile<bf16_t> { static constexpr int kStep = 16, kPitch = 68; };   // 136 B rows: 4 rows apart = 32 B mod 128
template <> struct XprojTile<float>  { static constexpr int kStep = 4,  kPitch = 80; };   // 320 B rows: 1 row apart = 64 B mod 128

typedef short short4v __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));

struct XprojArgs {
    const void* x; const void* Wx; const float* Wdt;
    void* delta_raw; void* Bm; void* Cm;
    int Dc, N, R, tiles;         // tiles per batch item
    long long P;                 // positions per map
};

template <typename T>
__global__ __launch_bounds__(256) void scan2d_block_xproj_kernel(const XprojArgs p) {
    constexpr int KS = XprojTile<T>::kStep, PT = XprojTile<T>::kPitch;
    constexpr int EB = Elem<T>::kBytes;
    using Raw = std::conditional_t<EB == 2, uint16_t, uint32_t>;
    extern __shared__ __align__(16) unsigned char smem[];
    const int Dc = p.Dc, N = p.N, R = p.R, M = R + 2 * N;
    const int DcP = (Dc + KS - 1) / KS * KS;
    Raw* xs = reinterpret_cast<Raw*>(smem);                                    // [DcP][PT]
    float* dtl = reinterpret_cast<float*>(smem + (size_t)DcP * PT * EB);       // [R][kTile]
    const int tid = threadIdx.x;
    const int b = blockIdx.x / p.tiles;
    const long long p0 = (long long)(blockIdx.x % p.tiles) * kTile;
    const long long P = p.P;
    const T* xb = static_cast<const T*>(p.x) + (size_t)b * Dc * P;
    const bool vec_ok = (P % 4) == 0;

    // ---- 1. the tile of x
    for (int idx = tid; idx < DcP * (kTile / 4); idx += 256) {
        const int c = idx / (kTile / 4), q = idx % (kTile / 4);
        const long long pos = p0 + 4 * q;
        Raw v[4] = {0, 0, 0, 0};
        if (c < Dc) {
            const T* src = xb + (size_t)c * P + pos;
            if (vec_ok && pos + 3 < P) {
                if constexpr (EB == 2) {
                    const uint2 t = *reinterpret_cast<const uint2*>(src);
                    v[0] = (Raw)(t.x & 0xffffu); v[1] = (Raw)(t.x >> 16); v[2] = (Raw)(t.y & 0xffffu); v[3] = (Raw)(t.y >> 16);
                } else {
                    const uint4 t = *reinterpret_cast<const uint4*>(src);
                    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (pos + e < P) v[e] = (Raw)elem_bits(src + e);
            }
        }
        Raw* dst = xs + (size_t)c * PT + 4 * q;
#pragma unroll
        for (int e = 0; e < 4; ++e) dst[e] = v[e];
    }
    __syncthreads();

    // ---- 2. low = Wx . x
    const int l = tid & 63, wv = tid >> 6, g = l >> 4, n = l & 15;
    const int ncol = wv * 16 + n;                         // position inside the tile
    const T* Wx = static_cast<const T*>(p.Wx);
    const bool wvec = (Dc % 4) == 0;
    const int MB = (M + 15) / 16;
    for (int m0 = 0; m0 < MB; m0 += 3) {
        float4v acc[3];
#pragma unroll
        for (int mb = 0; mb < 3; ++mb) acc[mb] = float4v{0.0f, 0.0f, 0.0f, 0.0f};
        for (int k0 = 0; k0 < DcP; k0 += KS) {
            if constexpr (EB == 2) {
                short4v bf;
                const Raw* col = xs + (size_t)(k0 + 4 * g) * PT + ncol;
                bf.x = (short)col[0]; bf.y = (short)col[PT]; bf.z = (short)col[2 * PT]; bf.w = (short)col[3 * PT];
#pragma unroll
                for (int mb = 0; mb < 3; ++mb) {
                    if (m0 + mb < MB) {
                        const int mrow = min((m0 + mb) * 16 + n, M - 1);       // rows past M are computed and dropped
                        const int k = k0 + 4 * g;
                        const T* src = Wx + (size_t)mrow * Dc + k;
                        short4v af;
                        if (wvec && k + 3 < Dc) {
                            const uint2 t = *reinterpret_cast<const uint2*>(src);
                            af.x = (short)(t.x & 0xffffu); af.y = (short)(t.x >> 16); af.z = (short)(t.y & 0xffffu); af.w = (short)(t.y >> 16);
                        } else {
                            af.x = k     < Dc ? (short)elem_bits(src)     : (short)0;
                            af.y = k + 1 < Dc ? (short)elem_bits(src + 1) : (short)0;
                            af.z = k + 2 < Dc ? (short)elem_bits(src + 2) : (short)0;
                            af.w = k + 3 < Dc ? (short)elem_bits(src + 3) : (short)0;
                        }
                        acc[mb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(af, bf, acc[mb], 0, 0, 0);
                    }
                }
            } else {
                const float bv = __uint_as_float(xs[(size_t)(k0 + g) * PT + ncol]);
#pragma unroll
                for (int mb = 0; mb < 3; ++mb) {
                    if (m0 + mb < MB) {
                        const int mrow = min((m0 + mb) * 16 + n, M - 1);
                        const int k = k0 + g;
                        const float av = k < Dc ? __uint_as_float(elem_bits(Wx + (size_t)mrow * Dc + k)) : 0.0f;
                        acc[mb] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv, acc[mb], 0, 0, 0);
                    }
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
    __syncthreads();

    // ---- 3. delta_raw = Wdt . low[:R]
    const int q = tid & 15;                               // positions 4q .. 4q+3 of the tile
    const long long pos = p0 + 4 * q;
    T* db = static_cast<T*>(p.delta_raw) + (size_t)b * Dc * P;
    for (int c = tid >> 4; c < Dc; c += 16) {
        const float* wr = p.Wdt + (size_t)c * R;
        float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
        for (int r = 0; r < R; ++r) {
            const float4 d = *reinterpret_cast<const float4*>(dtl + r * kTile + 4 * q);
            const float wv2 = wr[r];
            a0 = fmaf(wv2, d.x, a0); a1 = fmaf(wv2, d.y, a1); a2 = fmaf(wv2, d.z, a2); a3 = fmaf(wv2, d.w, a3);
        }
        T* dst = db + (size_t)c * P + pos;
        if (vec_ok && pos + 3 < P) {
            if constexpr (EB == 2) {
                uint2 o;
                o.x = f32_to_bf16_bits(a0) | (f32_to_bf16_bits(a1) << 16);
                o.y = f32_to_bf16_bits(a2) | (f32_to_bf16_bits(a3) << 16);
                *reinterpret_cast<uint2*>(dst) = o;
            } else {
                *reinterpret_cast<float4*>(dst) = make_float4(a0, a1, a2, a3);
            }
        } else {
            if (pos < P) store_elem(dst, a0);
            if (pos + 1 < P) store_elem(dst + 1, a1);
            if (pos + 2 < P) store_elem(dst + 2, a2);
            if (pos + 3 < P) store_elem(dst + 3, a3);
        }
    }
}

template <typename T>
size_t xproj_lds_bytes(int Dc, int R) {
    constexpr int KS = XprojTile<T>::kStep;
    const size_t DcP = (size_t)(Dc + KS - 1) / KS * KS;
    return DcP * XprojTile<T>::kPitch * Elem<T>::kBytes + (size_t)R * kTile * sizeof(float);
}

}  // namespace

bool allow_large_lds(const void* kernel, size_t bytes);   // scan2d_api.hip

int block_conv_silu_launch(const scan2d_desc* d, const scan2d_conv_shape* cs, const void* u, const float* w, const float* bias,
                           void* x, hipStream_t stream) {
    if (cs->KH < 1 || cs->KH > 7 || cs->KW < 1 || cs->KW > 7 || cs->PH < 0 || cs->PH >= cs->KH || cs->PW < 0 || cs->PW >= cs->KW)
        return SCAN2D_ERR_BAD_SHAPE;
    const long long maps = (long long)d->Bt * d->Dc;
    const long long total = maps * d->H * ((d->W + 3) / 4);
    const long long blocks = (total + 255) / 256;
    if (blocks > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
    (void)hipGetLastError();
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
    const size_t lds = bf16 ? xproj_lds_bytes<bf16_t>(d->Dc, R) : xproj_lds_bytes<float>(d->Dc, R);
    if (lds > 160 * 1024) return SCAN2D_ERR_BAD_SHAPE;           // Dc up to 1088 (bf16) / 448 (fp32) at R = 64
    XprojArgs a;
    a.x = x; a.Wx = Wx; a.Wdt = Wdt; a.delta_raw = delta_raw; a.Bm = Bm; a.Cm = Cm;
    a.Dc = d->Dc; a.N = d->N; a.R = R;
    a.P = (long long)d->H * d->W;
    const long long tiles = (a.P + kTile - 1) / kTile;
    if (tiles * d->Bt > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
    a.tiles = (int)tiles;
    (void)hipGetLastError();
    const void* kernel = bf16 ? reinterpret_cast<const void*>(scan2d_block_xproj_kernel<bf16_t>)
                              : reinterpret_cast<const void*>(scan2d_block_xproj_kernel<float>);
    if (lds > 65536 && !allow_large_lds(kernel, lds)) return SCAN2D_ERR_LAUNCH_FAILED;
    if (bf16) hipLaunchKernelGGL(scan2d_block_xproj_kernel<bf16_t>, dim3((unsigned)(tiles * d->Bt)), dim3(256), lds, stream, a);
    else hipLaunchKernelGGL(scan2d_block_xproj_kernel<float>, dim3((unsigned)(tiles * d->Bt)), dim3(256), lds, stream, a);
    return hipGetLastError() == hipSuccess ? SCAN2D_OK : SCAN2D_ERR_LAUNCH_FAILED;
}

}  // namespace scan2d
