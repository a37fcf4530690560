// The aggregator behind the last 2DMamba block (Supp. A "Aggregator": attention pooling with two linear layers):
//     s_k = sum_d w[d] * tanh(sum_m V[d,m] * h[m,k]),   a_k = softmax of s over the bag,   z = sum_k a_k h_k.
// Three kernels:
//   scan2d_pool_scores_kernel  : the scores.  V . h is a dense contraction (D x M x positions), so it runs on the matrix
//                                cores; tanh, the product with w and the sum over the D hidden units are its epilogue.
//   scan2d_pool_softmax_kernel : per batch item, max and sum of exp over the bag in a fixed order, then the weights.
//   scan2d_pool_sum_kernel     : z[b][m], one workgroup per channel, fixed order.
#include "scan2d_block.hpp"

#include <algorithm>

#include "scan2d_common.hpp"

namespace scan2d {
namespace {

typedef short short4v __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));

constexpr int kPoolTile = 64;        // positions per tile: 16 per wavefront
constexpr int kPoolRows = 128;       // hidden units, zero-padded: 8 MFMA row blocks
template <typename T> struct PoolTile;
// kChunk channels of V and of the tile of h are in LDS at a time; row pitches: the 16 lanes of a k-group that read one
// row each with a 64- or 128-bit load are 16 bytes apart mod 256, the four k-groups of the tile of h 64 bytes
template <> struct PoolTile<bf16_t> { static constexpr int kChunk = 128, kVPitch = 128 + 8, kXPitch = 68; };
template <> struct PoolTile<float>  { static constexpr int kChunk = 64,  kVPitch = 64 + 4,  kXPitch = 68; };

struct PoolArgs {
    const void* h; const void* V; const float* w; const uint8_t* mask;
    float* attn; float* z;
    int M, D, Bt, tiles;             // channels, hidden units, batch items, tiles per batch item
    long long P;                     // positions per map
};

__device__ __forceinline__ float fast_tanh(float v) {          // 1 - 2 / (1 + e^(2v)); saturates to +-1, keeps NaN
    return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(v * (2.0f * kLog2e)));
}

// Persistent workgroups of 4 wavefronts over tiles of 64 positions.  Everything the MFMA loop reads sits in LDS,
// zero-filled past M channels, D hidden units and the last position, so the loop carries no guard.  With at most one
// chunk of channels V goes to LDS once per workgroup.
// VEC: H*W and M are multiples of 4, so every group of 4 positions (of h) or 4 channels (of V) is one aligned vector
// that lies inside the tensor or outside it as a whole.
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void scan2d_pool_scores_kernel(const PoolArgs p) {
    constexpr int KC = PoolTile<T>::kChunk, VP = PoolTile<T>::kVPitch, XP = PoolTile<T>::kXPitch, NG = KC / 16;
    constexpr int EB = Elem<T>::kBytes;
    using Raw = std::conditional_t<EB == 2, uint16_t, uint32_t>;
    __shared__ __align__(16) Raw vL[kPoolRows * VP];
    __shared__ __align__(16) Raw xs[KC * XP];
    const int tid = threadIdx.x, l = tid & 63, wv = tid >> 6, g = l >> 4, n = l & 15;
    const int ncol = wv * 16 + n;
    const int M = p.M, D = p.D;
    const long long P = p.P;
    const T* V = static_cast<const T*>(p.V);
    const int NC = (M + KC - 1) / KC;

    float wr[8][4];                                       // w of the hidden units this lane's accumulators belong to
#pragma unroll
    for (int rb = 0; rb < 8; ++rb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int d = rb * 16 + 4 * g + i;
            const float v = p.w[min(d, D - 1)];
            wr[rb][i] = d < D ? v : 0.0f;
        }

    auto load_v = [&](int chunk) {                        // V[:, chunk] -> LDS, zero past D rows and M channels
        if constexpr (VEC) {
            using Vec = std::conditional_t<EB == 2, uint2, uint4>;
            constexpr int VPR = KC / 4, RPI = 256 / VPR;  // vectors per row, rows per iteration
            const int vq = tid % VPR, r0 = tid / VPR;
            const int c = chunk * KC + 4 * vq;
            Vec v[kPoolRows / RPI];
#pragma unroll
            for (int it = 0; it < kPoolRows / RPI; ++it) {
                const int d = r0 + it * RPI;
                const Vec t = *reinterpret_cast<const Vec*>(V + (size_t)min(d, D - 1) * M + min(c, M - 4));
                v[it] = (d < D && c < M) ? t : Vec{};
            }
#pragma unroll
            for (int it = 0; it < kPoolRows / RPI; ++it) *reinterpret_cast<Vec*>(vL + (size_t)(r0 + it * RPI) * VP + 4 * vq) = v[it];
        } else {
            constexpr int RPI = 256 / KC;                 // rows per iteration
            const int col = tid % KC, r0 = tid / KC;
            const int c = chunk * KC + col;
#pragma unroll 8
            for (int it = 0; it < kPoolRows / RPI; ++it) {
                const int d = r0 + it * RPI;
                const uint32_t bits = elem_bits(V + (size_t)min(d, D - 1) * M + min(c, M - 1));
                vL[d * VP + col] = (Raw)((d < D && c < M) ? bits : 0u);
            }
        }
    };
    if (NC == 1) load_v(0);

    const long long total = (long long)p.tiles * p.Bt;
    for (long long tile = blockIdx.x; tile < total; tile += gridDim.x) {
        const int b = (int)(tile / p.tiles);
        const long long p0 = (tile % p.tiles) * kPoolTile;
        const T* hb = static_cast<const T*>(p.h) + (size_t)b * M * P;
        float4v acc[8];
#pragma unroll
        for (int rb = 0; rb < 8; ++rb) acc[rb] = float4v{0.0f, 0.0f, 0.0f, 0.0f};
        for (int chunk = 0; chunk < NC; ++chunk) {
            __syncthreads();                              // the previous products have read both regions
            if (NC > 1) load_v(chunk);
            if constexpr (VEC) {
                using Vec = std::conditional_t<EB == 2, uint2, uint4>;
                const int cr0 = tid >> 4, q = tid & 15;
                const long long pp = p0 + 4 * q;
                const bool pin = pp < P;
                const T* src = hb + (size_t)min(pp, P - 4);
                Vec v[KC / 16];
#pragma unroll
                for (int it = 0; it < KC / 16; ++it) {
                    const int c = chunk * KC + cr0 + 16 * it;
                    const Vec t = *reinterpret_cast<const Vec*>(src + (size_t)min(c, M - 1) * P);
                    v[it] = (pin && c < M) ? t : Vec{};
                }
#pragma unroll
                for (int it = 0; it < KC / 16; ++it) *reinterpret_cast<Vec*>(xs + (size_t)(cr0 + 16 * it) * XP + 4 * q) = v[it];
            } else {
                const int pos = tid & 63, c0 = tid >> 6;
                const long long pp = p0 + pos;
                const bool pin = pp < P;
                const T* src = hb + (size_t)min(pp, P - 1);
#pragma unroll 8
                for (int it = 0; it < KC / 4; ++it) {
                    const int c = chunk * KC + c0 + 4 * it;
                    const uint32_t bits = elem_bits(src + (size_t)min(c, M - 1) * P);
                    xs[(c0 + 4 * it) * XP + pos] = (Raw)((pin && c < M) ? bits : 0u);
                }
            }
            __syncthreads();
#pragma unroll
            for (int kg = 0; kg < NG; ++kg) {
                const Raw* col = xs + (size_t)(kg * 16 + 4 * g) * XP + ncol;
                if constexpr (EB == 2) {
                    short4v bf;
                    bf.x = (short)col[0]; bf.y = (short)col[XP]; bf.z = (short)col[2 * XP]; bf.w = (short)col[3 * XP];
#pragma unroll
                    for (int rb = 0; rb < 8; ++rb) {
                        const uint2 t = *reinterpret_cast<const uint2*>(vL + (size_t)(rb * 16 + n) * VP + kg * 16 + 4 * g);
                        short4v af;
                        af.x = (short)(t.x & 0xffffu); af.y = (short)(t.x >> 16); af.z = (short)(t.y & 0xffffu); af.w = (short)(t.y >> 16);
                        acc[rb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(af, bf, acc[rb], 0, 0, 0);
                    }
                } else {
                    // the 16 channels of the group are contracted in the order (k-group of the lane, step) on both operands
                    const float b0 = __uint_as_float(col[0]), b1 = __uint_as_float(col[XP]);
                    const float b2 = __uint_as_float(col[2 * XP]), b3 = __uint_as_float(col[3 * XP]);
#pragma unroll
                    for (int rb = 0; rb < 8; ++rb) {
                        const float4 a = *reinterpret_cast<const float4*>(vL + (size_t)(rb * 16 + n) * VP + kg * 16 + 4 * g);
                        acc[rb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, b0, acc[rb], 0, 0, 0);
                        acc[rb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, b1, acc[rb], 0, 0, 0);
                        acc[rb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, b2, acc[rb], 0, 0, 0);
                        acc[rb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, b3, acc[rb], 0, 0, 0);
                    }
                }
            }
        }
        // ---- s = w . tanh(.): this lane holds hidden units rb*16 + 4g + i of position ncol
        float s = 0.0f;
#pragma unroll
        for (int rb = 0; rb < 8; ++rb)
#pragma unroll
            for (int i = 0; i < 4; ++i) s = fmaf(wr[rb][i], fast_tanh(acc[rb][i]), s);
        s += __shfl_xor(s, 16);
        s += __shfl_xor(s, 32);
        if (g == 0 && p0 + ncol < P) p.attn[(size_t)b * P + p0 + ncol] = s;
    }
}

constexpr int kSoftThreads = 1024;
// Sum or maximum over the workgroup in a fixed order; every thread gets the result.
template <bool MAX>
__device__ __forceinline__ float block_reduce(float v, float* red) {
    const int tid = threadIdx.x;
    red[tid] = v;
    __syncthreads();
    for (int step = kSoftThreads / 2; step > 0; step >>= 1) {
        if (tid < step) red[tid] = MAX ? fmaxf(red[tid], red[tid + step]) : red[tid] + red[tid + step];
        __syncthreads();
    }
    const float r = red[0];
    __syncthreads();
    return r;
}

// One workgroup per batch item, in place: scores -> attention weights.  Positions under the mask are not members of
// the bag: they are skipped by the maximum and the sum and get weight 0; an empty bag gets all zeros.  Every thread
// walks its positions four loads deep (VEC: four aligned groups of 4 positions), in an order fixed by the shape.
template <bool VEC>
__global__ __launch_bounds__(kSoftThreads) void scan2d_pool_softmax_kernel(const PoolArgs p) {
    __shared__ float red[kSoftThreads];
    constexpr int E = VEC ? 4 : 1;                        // positions per load
    const int b = blockIdx.x, tid = threadIdx.x;
    const long long P = p.P, PV = P / E;
    float* a = p.attn + (size_t)b * P;
    const uint8_t* mk = p.mask ? p.mask + (size_t)b * P : nullptr;
    // pass(f): f(position, score, member) over this thread's positions
    auto walk = [&](auto f) {
        for (long long base = 0; base < PV; base += 4 * kSoftThreads) {
            float sv[4][E];
            uint32_t mv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const long long idx = min(base + u * kSoftThreads + tid, PV - 1);
                if constexpr (VEC) {
                    const float4 t = *reinterpret_cast<const float4*>(a + 4 * idx);
                    sv[u][0] = t.x; sv[u][1] = t.y; sv[u][2] = t.z; sv[u][3] = t.w;
                    mv[u] = mk ? *reinterpret_cast<const uint32_t*>(mk + 4 * idx) : 0u;
                } else {
                    sv[u][0] = a[idx];
                    mv[u] = mk ? (uint32_t)mk[idx] : 0u;
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const long long idx = base + u * kSoftThreads + tid;
                if (idx < PV) {
#pragma unroll
                    for (int e = 0; e < E; ++e) f(E * idx + e, sv[u][e], ((mv[u] >> (8 * e)) & 0xffu) == 0u);
                }
            }
        }
    };
    float mx = -INFINITY;
    walk([&](long long, float s, bool member) { mx = member ? fmaxf(mx, s) : mx; });
    mx = block_reduce<true>(mx, red);
    float sum = 0.0f;
    walk([&](long long, float s, bool member) { sum += member ? __builtin_amdgcn_exp2f((s - mx) * kLog2e) : 0.0f; });
    sum = block_reduce<false>(sum, red);
    const float inv = sum > 0.0f ? 1.0f / sum : 0.0f;     // a NaN score makes the sum NaN: the weights then are NaN too
    const bool bad = sum != sum;
    walk([&](long long k, float s, bool member) {
        const float e = __builtin_amdgcn_exp2f((s - mx) * kLog2e);
        a[k] = member ? (bad ? sum : e * inv) : 0.0f;
    });
}

// z[b][m] = sum over the bag of a_k * h[m][k]: grid (M, Bt), fixed order (strided partial sums four loads deep, then a
// tree over the workgroup).
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void scan2d_pool_sum_kernel(const PoolArgs p) {
    __shared__ float red[256];
    constexpr int E = VEC ? 4 : 1, EB = Elem<T>::kBytes;
    const int m = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const long long P = p.P, PV = P / E;
    const T* hr = static_cast<const T*>(p.h) + ((size_t)b * p.M + m) * P;
    const float* a = p.attn + (size_t)b * P;
    float acc = 0.0f;
    for (long long base = 0; base < PV; base += 4 * 256) {
        float av[4][E], hv[4][E];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const long long idx = min(base + u * 256 + tid, PV - 1);
            if constexpr (VEC) {
                const float4 t = *reinterpret_cast<const float4*>(a + 4 * idx);
                av[u][0] = t.x; av[u][1] = t.y; av[u][2] = t.z; av[u][3] = t.w;
                if constexpr (EB == 2) {
                    const uint2 r = *reinterpret_cast<const uint2*>(hr + 4 * idx);
                    hv[u][0] = __uint_as_float(r.x << 16); hv[u][1] = __uint_as_float(r.x & 0xffff0000u);
                    hv[u][2] = __uint_as_float(r.y << 16); hv[u][3] = __uint_as_float(r.y & 0xffff0000u);
                } else {
                    const float4 r = *reinterpret_cast<const float4*>(hr + 4 * idx);
                    hv[u][0] = r.x; hv[u][1] = r.y; hv[u][2] = r.z; hv[u][3] = r.w;
                }
            } else {
                av[u][0] = a[idx];
                const uint32_t bits = elem_bits(hr + idx);
                hv[u][0] = EB == 4 ? __uint_as_float(bits) : __uint_as_float(bits << 16);
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (base + u * 256 + tid < PV) {
#pragma unroll
                for (int e = 0; e < E; ++e) acc += av[u][e] != 0.0f ? av[u][e] * hv[u][e] : 0.0f;   // weight 0: outside the bag, never read into the sum
            }
        }
    }
    red[tid] = acc;
    __syncthreads();
    for (int step = 128; step > 0; step >>= 1) {
        if (tid < step) red[tid] += red[tid + step];
        __syncthreads();
    }
    if (tid == 0) p.z[(size_t)b * p.M + m] = red[0];
}

}  // namespace

int block_attn_pool_launch(const scan2d_desc* d, int D, const void* h, const void* V, const float* w, const uint8_t* mask,
                           float* attn, float* z, hipStream_t stream) {
    if (D < 1 || D > kPoolRows) return SCAN2D_ERR_BAD_SHAPE;
    PoolArgs a;
    a.h = h; a.V = V; a.w = w; a.mask = mask; a.attn = attn; a.z = z;
    a.M = d->Dc; a.D = D; a.Bt = d->Bt;
    a.P = (long long)d->H * d->W;
    const long long tiles = (a.P + kPoolTile - 1) / kPoolTile;
    if (tiles * d->Bt > 2147483647LL || d->Bt > 65535) return SCAN2D_ERR_BAD_SHAPE;
    a.tiles = (int)tiles;
    const bool bf16 = d->dtype == SCAN2D_BF16;
    (void)hipGetLastError();
    const long long grid = std::min<long long>(tiles * d->Bt, 2 * 256);       // persistent: V is staged once per workgroup
    const bool vec = a.P % 4 == 0 && a.M % 4 == 0;
    const dim3 g1((unsigned)grid), g2((unsigned)d->Bt), g3((unsigned)d->Dc, (unsigned)d->Bt);
#define SCAN2D_POOL_LAUNCH(T, VEC)                                                                        \
    do {                                                                                                  \
        hipLaunchKernelGGL((scan2d_pool_scores_kernel<T, VEC>), g1, dim3(256), 0, stream, a);             \
        hipLaunchKernelGGL(scan2d_pool_softmax_kernel<VEC>, g2, dim3(kSoftThreads), 0, stream, a);        \
        hipLaunchKernelGGL((scan2d_pool_sum_kernel<T, VEC>), g3, dim3(256), 0, stream, a);                \
    } while (0)
    if (bf16) { if (vec) SCAN2D_POOL_LAUNCH(bf16_t, true); else SCAN2D_POOL_LAUNCH(bf16_t, false); }
    else { if (vec) SCAN2D_POOL_LAUNCH(float, true); else SCAN2D_POOL_LAUNCH(float, false); }
#undef SCAN2D_POOL_LAUNCH
    return hipGetLastError() == hipSuccess ? SCAN2D_OK : SCAN2D_ERR_LAUNCH_FAILED;
}

}  // namespace scan2d
