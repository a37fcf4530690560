// The normalisation in front of a 2DMamba block (Sec. 3.3 lists "normalization, projection, and convolution" in front of
// the scan) on channel-major maps, over the channels of each position:
//     layer norm: out = (x - mean_c x) / sqrt(var_c x + eps) * gamma[c] + beta[c]      (biased variance)
//     RMS norm:   out = x / sqrt(mean_c x^2 + eps) * gamma[c] (+ beta[c])
// HBM-bound (one read, one write per element; the second and third pass over a workgroup's tile come from L2).  A
// workgroup owns 32 groups of E consecutive positions (E = 4 when H*W is a multiple of 4, else 1); its threads split the
// channels eight ways (half-wavefront s takes channels s, s + 8, ...), so every load is a row segment of 32 vectors,
// eight loads in flight per thread, and the per-position sums of the eight parts meet in LDS in a fixed order.  The
// mean is taken first and the variance as the mean of squared deviations (no cancellation), then the tile is read a
// third time and written.
#include "scan2d_block.hpp"

#include "scan2d_common.hpp"

namespace scan2d {
namespace {

typedef float float2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack2_bf16_norm(float lo, float hi) {  // nearest even, one v_cvt_pk_bf16_f32
    const float2v v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2v));
}

struct NormArgs {
    const void* in; const float* gamma; const float* beta; void* out;
    int C, Bt, rms;
    float eps;
    long long P, groups;            // positions per map, groups of E positions per map
};

constexpr int kNormGroups = 32, kNormSplit = 8, kNormDeep = 8;   // position groups and channel parts per workgroup, loads in flight
static_assert(kNormGroups * kNormSplit == 256, "one thread per (position group, channel part)");
template <typename T, int E>
__global__ __launch_bounds__(256) void scan2d_norm_kernel(const NormArgs p) {
    constexpr int EB = Elem<T>::kBytes;
    __shared__ float red[kNormSplit][kNormGroups][E];
    const int tid = threadIdx.x, q = tid % kNormGroups, cq = tid / kNormGroups;
    const long long per_item = (p.groups + kNormGroups - 1) / kNormGroups; // workgroups per batch item
    const int b = (int)(blockIdx.x / per_item);
    const long long grp = (blockIdx.x % per_item) * kNormGroups + q;
    const bool live = grp < p.groups;
    const long long pos = min(grp, p.groups - 1) * E;
    const int C = p.C;
    const T* src = static_cast<const T*>(p.in) + (size_t)b * C * p.P + pos;
    T* dst = static_cast<T*>(p.out) + (size_t)b * C * p.P + pos;

    auto load = [&](int c, float* v) {
        const T* a = src + (size_t)c * p.P;
        if constexpr (E == 4 && EB == 2) {
            const uint2 r = *reinterpret_cast<const uint2*>(a);
            v[0] = __uint_as_float(r.x << 16); v[1] = __uint_as_float(r.x & 0xffff0000u);
            v[2] = __uint_as_float(r.y << 16); v[3] = __uint_as_float(r.y & 0xffff0000u);
        } else if constexpr (E == 4) {
            const float4 r = *reinterpret_cast<const float4*>(a);
            v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w;
        } else {
            const uint32_t bits = elem_bits(a);
            v[0] = EB == 4 ? __uint_as_float(bits) : __uint_as_float(bits << 16);
        }
    };
    // sum over all channels of f(x) per position: this thread's channels kNormDeep loads deep, then the partial sums
    auto channel_sum = [&](auto f, float* total) {
        float acc[E];
#pragma unroll
        for (int e = 0; e < E; ++e) acc[e] = 0.0f;
        for (int c0 = cq; c0 < C; c0 += kNormSplit * kNormDeep) {
            float v[kNormDeep][E];
#pragma unroll
            for (int u = 0; u < kNormDeep; ++u) load(min(c0 + kNormSplit * u, C - 1), v[u]);
#pragma unroll
            for (int u = 0; u < kNormDeep; ++u)
                if (c0 + kNormSplit * u < C) {
#pragma unroll
                    for (int e = 0; e < E; ++e) acc[e] += f(v[u][e], e);
                }
        }
        __syncthreads();                                   // the previous sums have been read
#pragma unroll
        for (int e = 0; e < E; ++e) red[cq][q][e] = acc[e];
        __syncthreads();
#pragma unroll
        for (int e = 0; e < E; ++e) {
            float t2 = 0.0f;
#pragma unroll
            for (int s = 0; s < kNormSplit; ++s) t2 += red[s][q][e];
            total[e] = t2;
        }
    };

    float mean[E], rstd[E], t[E];
#pragma unroll
    for (int e = 0; e < E; ++e) mean[e] = 0.0f;
    const float invC = 1.0f / (float)C;
    if (!p.rms) {
        channel_sum([](float x, int) { return x; }, t);
#pragma unroll
        for (int e = 0; e < E; ++e) mean[e] = t[e] * invC;
    }
    channel_sum([&](float x, int e) { const float d = x - mean[e]; return d * d; }, t);
#pragma unroll
    for (int e = 0; e < E; ++e) rstd[e] = 1.0f / sqrtf(t[e] * invC + p.eps);

    for (int c0 = cq; c0 < C; c0 += kNormSplit * kNormDeep) {
        float v[kNormDeep][E];
#pragma unroll
        for (int u = 0; u < kNormDeep; ++u) load(min(c0 + kNormSplit * u, C - 1), v[u]);
#pragma unroll
        for (int u = 0; u < kNormDeep; ++u) {
            const int c = c0 + kNormSplit * u;
            if (c < C && live) {
                const float gm = p.gamma[c], bt = p.beta ? p.beta[c] : 0.0f;
                float o[E];
#pragma unroll
                for (int e = 0; e < E; ++e) o[e] = fmaf((v[u][e] - mean[e]) * rstd[e], gm, bt);
                T* d = dst + (size_t)c * p.P;
                if constexpr (E == 4 && EB == 2) {
                    uint2 r;
                    r.x = pack2_bf16_norm(o[0], o[1]); r.y = pack2_bf16_norm(o[2], o[3]);
                    *reinterpret_cast<uint2*>(d) = r;
                } else if constexpr (E == 4) {
                    *reinterpret_cast<float4*>(d) = make_float4(o[0], o[1], o[2], o[3]);
                } else {
                    store_elem(d, o[0]);
                }
            }
        }
    }
}

}  // namespace

int block_norm_launch(const scan2d_desc* d, int kind, float eps, const void* in, const float* gamma, const float* beta, void* out,
                      hipStream_t stream) {
    if ((kind != 0 && kind != 1) || !(eps >= 0.0f)) return SCAN2D_ERR_BAD_SHAPE;
    NormArgs a;
    a.in = in; a.gamma = gamma; a.beta = beta; a.out = out;
    a.C = d->Dc; a.Bt = d->Bt; a.rms = kind; a.eps = eps;
    a.P = (long long)d->H * d->W;
    const bool vec = a.P % 4 == 0;
    a.groups = vec ? a.P / 4 : a.P;
    const long long blocks = (a.groups + kNormGroups - 1) / kNormGroups * d->Bt;
    if (blocks > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
    const bool bf16 = d->dtype == SCAN2D_BF16;
    (void)hipGetLastError();
    if (bf16) {
        if (vec) hipLaunchKernelGGL((scan2d_norm_kernel<bf16_t, 4>), dim3((unsigned)blocks), dim3(256), 0, stream, a);
        else hipLaunchKernelGGL((scan2d_norm_kernel<bf16_t, 1>), dim3((unsigned)blocks), dim3(256), 0, stream, a);
    } else {
        if (vec) hipLaunchKernelGGL((scan2d_norm_kernel<float, 4>), dim3((unsigned)blocks), dim3(256), 0, stream, a);
        else hipLaunchKernelGGL((scan2d_norm_kernel<float, 1>), dim3((unsigned)blocks), dim3(256), 0, stream, a);
    }
    return hipGetLastError() == hipSuccess ? SCAN2D_OK : SCAN2D_ERR_LAUNCH_FAILED;
}

}  // namespace scan2d
