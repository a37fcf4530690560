// Roofline probe for the box the benchmark runs on: achievable HBM bandwidth (copy and
// read-only kernels of known size), fp32 vector issue rates (FMA, add, v_exp_f32; a short loop of 8
// operations and an unrolled stream of 256) against the number of waves per CU, and the launch overhead.  Stand-alone executable:
//     roofprobe            all measurements
//     roofprobe --copy N   only N launches of the 1 GiB copy kernel (counter calibration:
//                          each launch reads 2^30 bytes and writes 2^30 bytes)
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 1; } } while (0)

__global__ void k_fma(float* out, int iters, float s) {
    float a0 = threadIdx.x, a1 = a0 + 1, a2 = a0 + 2, a3 = a0 + 3, a4 = a0 + 4, a5 = a0 + 5, a6 = a0 + 6, a7 = a0 + 7;
    for (int i = 0; i < iters; ++i) {
        a0 = fmaf(a0, s, 1.f); a1 = fmaf(a1, s, 1.f); a2 = fmaf(a2, s, 1.f); a3 = fmaf(a3, s, 1.f);
        a4 = fmaf(a4, s, 1.f); a5 = fmaf(a5, s, 1.f); a6 = fmaf(a6, s, 1.f); a7 = fmaf(a7, s, 1.f);
    }
    out[blockIdx.x * blockDim.x + threadIdx.x] = a0 + a1 + a2 + a3 + a4 + a5 + a6 + a7;
}
// The same with 256 FMAs per trip: 16 independent chains (DEP = false) or one dependent chain (DEP = true).  A wave
// that is alone on its SIMD pays for the loop control of the short loop above in full; here it issues back to back.
template <bool DEP>
__global__ void k_fma_unrolled(float* out, int iters, float s) {
    float a[16];
    for (int i = 0; i < 16; ++i) a[i] = threadIdx.x + i;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 16; ++u)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if (DEP) a[0] = fmaf(a[0], s, 1.f);
                else a[i] = fmaf(a[i], s, 1.f);
            }
    }
    float t = 0;
    for (int i = 0; i < 16; ++i) t += a[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = t;
}
__global__ void k_add(float* out, int iters, float s) {
    float a0 = threadIdx.x * 1e-3f, a1 = a0 + .1f, a2 = a0 + .2f, a3 = a0 + .3f, a4 = a0 + .4f, a5 = a0 + .5f, a6 = a0 + .6f, a7 = a0 + .7f;
    for (int i = 0; i < iters; ++i) { a0 -= s; a1 -= s; a2 -= s; a3 -= s; a4 -= s; a5 -= s; a6 -= s; a7 -= s; }
    out[blockIdx.x * blockDim.x + threadIdx.x] = a0 + a1 + a2 + a3 + a4 + a5 + a6 + a7;
}
__global__ void k_exp(float* out, int iters) {
    float a0 = threadIdx.x * 1e-3f, a1 = a0 + .1f, a2 = a0 + .2f, a3 = a0 + .3f, a4 = a0 + .4f, a5 = a0 + .5f, a6 = a0 + .6f, a7 = a0 + .7f;
    for (int i = 0; i < iters; ++i) {   // 8 v_exp_f32 + 8 subtractions that keep the values bounded
        a0 = __builtin_amdgcn_exp2f(a0) - 1.f; a1 = __builtin_amdgcn_exp2f(a1) - 1.f;
        a2 = __builtin_amdgcn_exp2f(a2) - 1.f; a3 = __builtin_amdgcn_exp2f(a3) - 1.f;
        a4 = __builtin_amdgcn_exp2f(a4) - 1.f; a5 = __builtin_amdgcn_exp2f(a5) - 1.f;
        a6 = __builtin_amdgcn_exp2f(a6) - 1.f; a7 = __builtin_amdgcn_exp2f(a7) - 1.f;
    }
    out[blockIdx.x * blockDim.x + threadIdx.x] = a0 + a1 + a2 + a3 + a4 + a5 + a6 + a7;
}
__global__ void k_copy(const float4* __restrict__ in, float4* __restrict__ out, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) out[i] = in[i];
}
__global__ void k_read(const float4* __restrict__ in, float* out, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    float s = 0;
    for (; i < n; i += stride) { const float4 v = in[i]; s += v.x + v.y + v.z + v.w; }
    if (s == 12345.678f) out[0] = s;
}

template <class F> static float time_ms(F f, int reps) {
    hipEvent_t a, b;
    (void)hipEventCreate(&a); (void)hipEventCreate(&b);
    f(); (void)hipDeviceSynchronize();
    (void)hipEventRecord(a);
    for (int i = 0; i < reps; ++i) f();
    (void)hipEventRecord(b); (void)hipEventSynchronize(b);
    float ms = 0; (void)hipEventElapsedTime(&ms, a, b);
    return ms / reps;
}

int main(int argc, char** argv) {
    hipDeviceProp_t p;
    CK(hipGetDeviceProperties(&p, 0));
    const int CUs = p.multiProcessorCount;
    const size_t n = (size_t)1 << 26;   // float4 elements: 1 GiB
    float4 *a, *b;
    float* out;
    CK(hipMalloc(&a, n * 16)); CK(hipMalloc(&b, n * 16)); CK(hipMalloc(&out, (size_t)CUs * 16 * 256 * 4));
    CK(hipMemset(a, 1, n * 16));
    if (argc >= 3 && std::strcmp(argv[1], "--copy") == 0) {
        const int reps = std::atoi(argv[2]);
        for (int i = 0; i < reps; ++i) k_copy<<<CUs * 4, 256>>>(a, b, n);
        CK(hipDeviceSynchronize());
        std::printf("copy kernel: %d launches, each reads %zu bytes and writes %zu bytes\n", reps, n * 16, n * 16);
        return 0;
    }
    std::printf("device %s, %d CUs, clock %d kHz, LDS per workgroup %zu bytes\n", p.gcnArchName, CUs, p.clockRate, p.sharedMemPerBlock);
    const int iters = 20000;
    for (int wpc : {4, 8, 16, 32}) {   // waves per CU
        dim3 g(CUs * wpc / 4), t(256);
        const double lanes = (double)g.x * 256;
        const float f = time_ms([&] { k_fma<<<g, t>>>(out, iters, 0.999f); }, 3);
        const float ad = time_ms([&] { k_add<<<g, t>>>(out, iters, 0.001f); }, 3);
        const float ex = time_ms([&] { k_exp<<<g, t>>>(out, iters); }, 3);
        const int ui = iters / 20;
        const float fu = time_ms([&] { k_fma_unrolled<false><<<g, t>>>(out, ui, 0.999f); }, 3);
        const float fd = time_ms([&] { k_fma_unrolled<true><<<g, t>>>(out, ui, 0.999f); }, 3);
        std::printf("waves/CU %2d: fma %.2f T lane-op/s, add %.2f T lane-op/s, exp2+sub pair takes %.2f add slots (v_exp_f32 ~ %.2f slots)\n",
                    wpc, lanes * iters * 8 / f / 1e9, lanes * iters * 8 / ad / 1e9, ex / ad, ex / ad - 1.0);
        std::printf("             256 FMAs per loop trip: %.2f T lane-op/s in 16 independent chains, %.2f T in one dependent chain\n",
                    lanes * ui * 256 / fu / 1e9, lanes * ui * 256 / fd / 1e9);
    }
    for (int blocks : {CUs * 4, CUs * 8, CUs * 16}) {
        const float c = time_ms([&] { k_copy<<<blocks, 256>>>(a, b, n); }, 5);
        const float r = time_ms([&] { k_read<<<blocks, 256>>>(a, out, n); }, 5);
        std::printf("blocks %5d: copy 1 GiB -> 1 GiB %.3f ms = %.0f GB/s (read + write), read-only %.3f ms = %.0f GB/s\n",
                    blocks, c, 2.0 * n * 16 / c / 1e6, r, 1.0 * n * 16 / r / 1e6);
    }
    const float l = time_ms([&] { k_copy<<<1, 64>>>(a, b, 1); }, 200);
    std::printf("back-to-back launch of a trivial kernel: %.2f us\n", l * 1e3);
    return 0;
}
