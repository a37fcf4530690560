// Element-wise kernels beside the scan kernels (see scan2d_elementwise.hpp).
#include "scan2d_elementwise.hpp"

#include <algorithm>

#include "scan2d_common.hpp"

namespace scan2d {
namespace {

// y = y_scan * SiLU(z); four consecutive elements per thread and trip.
template <typename T>
__global__ __launch_bounds__(256) void scan2d_gate_fwd_kernel(const T* __restrict__ ys, const T* __restrict__ z, T* __restrict__ y, size_t n) {
    constexpr int XW = words_of<T, 4>();
    const size_t quads = n / 4;
    for (size_t q = (size_t)blockIdx.x * blockDim.x + threadIdx.x; q < quads; q += (size_t)gridDim.x * blockDim.x) {
        uint32_t rz[XW], ry[XW], o[XW];
        load_words<XW>(reinterpret_cast<const uint32_t*>(z + 4 * q), rz);
        load_words<XW>(reinterpret_cast<const uint32_t*>(ys + 4 * q), ry);
#pragma unroll
        for (int w = 0; w < XW; ++w) o[w] = 0u;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float zv = get_elem<T, 4>(rz, j);
            put_elem<T, 4>(o, j, to_elem_bits<T>(get_elem<T, 4>(ry, j) * (zv * logistic_f32(zv))));
        }
        store_words<XW>(reinterpret_cast<uint32_t*>(y + 4 * q), o);
    }
    if (blockIdx.x == 0 && threadIdx.x < n - 4 * quads) {                 // the last n % 4 elements
        const size_t e = 4 * quads + threadIdx.x;
        float zv, yv;
        if constexpr (Elem<T>::kBytes == 4) { zv = __uint_as_float(elem_bits(z + e)); yv = __uint_as_float(elem_bits(ys + e)); }
        else { zv = __uint_as_float(elem_bits(z + e) << 16); yv = __uint_as_float(elem_bits(ys + e) << 16); }
        store_elem(y + e, yv * (zv * logistic_f32(zv)));
    }
}

// Output gate: dyg = dy * SiLU(z), dz = dy * y_scan * s (1 + z (1 - s)) with s = 1 / (1 + exp(-z));
// four consecutive elements per thread and trip.
template <typename T>
__global__ __launch_bounds__(256) void scan2d_gate_bwd_kernel(const T* __restrict__ z, const T* __restrict__ ys, const T* __restrict__ dy,
                                                              T* __restrict__ dyg, T* __restrict__ dz, size_t n) {
    constexpr int XW = words_of<T, 4>();
    const size_t quads = n / 4;
    for (size_t q = (size_t)blockIdx.x * blockDim.x + threadIdx.x; q < quads; q += (size_t)gridDim.x * blockDim.x) {
        uint32_t rz[XW], ry[XW], rd[XW], og[XW], oz[XW];
        load_words<XW>(reinterpret_cast<const uint32_t*>(z + 4 * q), rz);
        load_words<XW>(reinterpret_cast<const uint32_t*>(ys + 4 * q), ry);
        load_words<XW>(reinterpret_cast<const uint32_t*>(dy + 4 * q), rd);
#pragma unroll
        for (int w = 0; w < XW; ++w) { og[w] = 0u; oz[w] = 0u; }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float zv = get_elem<T, 4>(rz, j), yv = get_elem<T, 4>(ry, j), dv = get_elem<T, 4>(rd, j);
            const float s = logistic_f32(zv);
            put_elem<T, 4>(og, j, to_elem_bits<T>(dv * (zv * s)));
            put_elem<T, 4>(oz, j, to_elem_bits<T>(dv * yv * (s * fmaf(zv, 1.0f - s, 1.0f))));
        }
        store_words<XW>(reinterpret_cast<uint32_t*>(dyg + 4 * q), og);
        store_words<XW>(reinterpret_cast<uint32_t*>(dz + 4 * q), oz);
    }
    if (blockIdx.x == 0 && threadIdx.x < n - 4 * quads) {                 // the last n % 4 elements
        const size_t e = 4 * quads + threadIdx.x;
        float zv, yv, dv;
        if constexpr (Elem<T>::kBytes == 4) {
            zv = __uint_as_float(elem_bits(z + e)); yv = __uint_as_float(elem_bits(ys + e)); dv = __uint_as_float(elem_bits(dy + e));
        } else {
            zv = __uint_as_float(elem_bits(z + e) << 16); yv = __uint_as_float(elem_bits(ys + e) << 16); dv = __uint_as_float(elem_bits(dy + e) << 16);
        }
        const float s = logistic_f32(zv);
        store_elem(dyg + e, dv * (zv * s));
        store_elem(dz + e, dv * yv * (s * fmaf(zv, 1.0f - s, 1.0f)));
    }
}


// out = mask ? fill : delta for one map per blockIdx.y-like chunk: map = blockIdx.x / chunks, 1024 positions per workgroup.
template <typename T>
__global__ __launch_bounds__(256) void scan2d_skip_step_kernel(const T* __restrict__ delta, const uint8_t* __restrict__ mask,
                                                               T* __restrict__ out, size_t HW, int Dc, unsigned chunks, uint32_t fill_bits) {
    const size_t map = blockIdx.x / chunks;
    const uint8_t* m = mask + (map / Dc) * HW;
    const T* src = delta + map * HW;
    T* dst = out + map * HW;
    const size_t e0 = ((size_t)(blockIdx.x % chunks) * 256 + threadIdx.x) * 4;
    if (e0 + 4 <= HW && (Elem<T>::kBytes == 4 || (HW & 1) == 0)) {      // four elements at once (maps stay 4-byte aligned)
        constexpr int XW = words_of<T, 4>();
        uint32_t r[XW], o[XW];
        load_words<XW>(reinterpret_cast<const uint32_t*>(src + e0), r);
#pragma unroll
        for (int w = 0; w < XW; ++w) o[w] = 0u;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t bits;
            if constexpr (Elem<T>::kBytes == 4) bits = r[j]; else bits = (r[j >> 1] >> (16 * (j & 1))) & 0xffffu;
            put_elem<T, 4>(o, j, m[e0 + j] != 0 ? fill_bits : bits);
        }
        store_words<XW>(reinterpret_cast<uint32_t*>(dst + e0), o);
        return;
    }
    for (size_t e = e0; e < e0 + 4 && e < HW; ++e) {
        T v = src[e];
        if (m[e] != 0) {
            if constexpr (Elem<T>::kBytes == 4) v = __uint_as_float(fill_bits);
            else v.bits = static_cast<uint16_t>(fill_bits);
        }
        dst[e] = v;
    }
}
// ddelta = 0 under the mask.
template <typename T>
__global__ __launch_bounds__(256) void scan2d_skip_grad_kernel(const uint8_t* __restrict__ mask, T* __restrict__ ddelta,
                                                               size_t HW, int Dc, unsigned chunks) {
    const size_t map = blockIdx.x / chunks;
    const uint8_t* m = mask + (map / Dc) * HW;
    T* dst = ddelta + map * HW;
    const size_t e0 = ((size_t)(blockIdx.x % chunks) * 256 + threadIdx.x) * 4;
    for (size_t e = e0; e < e0 + 4 && e < HW; ++e) {
        if (m[e] != 0) {
            if constexpr (Elem<T>::kBytes == 4) dst[e] = 0.0f;
            else dst[e].bits = 0;
        }
    }
}

// dst[p][j][i] = src[p][i][j]; one workgroup (32 x 8 threads) per 32 x 32 tile, tiles of all planes in one 1D grid.
template <typename E>
__global__ __launch_bounds__(256) void scan2d_transpose_kernel(const E* __restrict__ src, E* __restrict__ dst, int H, int W,
                                                               unsigned tiles_w, unsigned tiles_h) {
    __shared__ E tile[32][33];
    const unsigned per = tiles_w * tiles_h;
    const size_t plane = blockIdx.x / per;
    const unsigned rem = blockIdx.x % per, th = rem / tiles_w, tw = rem % tiles_w;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const E* s = src + plane * (size_t)H * W;
    E* d = dst + plane * (size_t)H * W;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int row = (int)th * 32 + ty + 8 * k, col = (int)tw * 32 + tx;
        if (row < H && col < W) tile[ty + 8 * k][tx] = s[(size_t)row * W + col];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int orow = (int)tw * 32 + ty + 8 * k, ocol = (int)th * 32 + tx;      // row of dst = column of src
        if (orow < W && ocol < H) d[(size_t)orow * H + ocol] = tile[tx][ty + 8 * k];
    }
}

unsigned gate_blocks(size_t n) { return (unsigned)std::min<size_t>((n / 4 + 255) / 256 + 1, 256 * 16); }

}  // namespace

int gate_fwd_launch(const scan2d_desc* d, const void* y_scan, const void* z, void* y, hipStream_t stream) {
    const size_t n = (size_t)d->Bt * d->Dc * d->H * d->W;
    (void)hipGetLastError();
    if (d->dtype == SCAN2D_BF16)
        hipLaunchKernelGGL(scan2d_gate_fwd_kernel<bf16_t>, dim3(gate_blocks(n)), dim3(256), 0, stream,
                           static_cast<const bf16_t*>(y_scan), static_cast<const bf16_t*>(z), static_cast<bf16_t*>(y), n);
    else
        hipLaunchKernelGGL(scan2d_gate_fwd_kernel<float>, dim3(gate_blocks(n)), dim3(256), 0, stream,
                           static_cast<const float*>(y_scan), static_cast<const float*>(z), static_cast<float*>(y), n);
    return hipGetLastError() == hipSuccess ? SCAN2D_OK : SCAN2D_ERR_LAUNCH_FAILED;
}

size_t gate_bwd_bytes(const scan2d_desc* d) {
    const size_t bytes = (size_t)d->Bt * d->Dc * d->H * d->W * (d->dtype == SCAN2D_BF16 ? 2 : 4);
    return (bytes + 255) & ~(size_t)255;
}

int gate_bwd_launch(const scan2d_desc* d, const void* z, const void* y_scan, const void* dy, void* dyg, void* dz,
                    hipStream_t stream) {
    const size_t n = (size_t)d->Bt * d->Dc * d->H * d->W;
    (void)hipGetLastError();
    if (d->dtype == SCAN2D_BF16)
        hipLaunchKernelGGL(scan2d_gate_bwd_kernel<bf16_t>, dim3(gate_blocks(n)), dim3(256), 0, stream, static_cast<const bf16_t*>(z),
                           static_cast<const bf16_t*>(y_scan), static_cast<const bf16_t*>(dy), static_cast<bf16_t*>(dyg),
                           static_cast<bf16_t*>(dz), n);
    else
        hipLaunchKernelGGL(scan2d_gate_bwd_kernel<float>, dim3(gate_blocks(n)), dim3(256), 0, stream, static_cast<const float*>(z),
                           static_cast<const float*>(y_scan), static_cast<const float*>(dy), static_cast<float*>(dyg),
                           static_cast<float*>(dz), n);
    return hipGetLastError() == hipSuccess ? SCAN2D_OK : SCAN2D_ERR_LAUNCH_FAILED;
}

size_t skip_bytes(const scan2d_desc* d) {
    if ((d->flags & SCAN2D_FLAG_IDENTITY_CELLS) == 0) return 0;
    return gate_bwd_bytes(d);                      // one tensor of the storage type, rounded up to 256 bytes
}

int skip_step_launch(const scan2d_desc* d, const void* delta, const uint8_t* mask, bool minus_inf, void* out, hipStream_t stream) {
    const size_t HW = (size_t)d->H * d->W;
    const long long maps = (long long)d->Bt * d->Dc;
    const unsigned chunks = (unsigned)((HW + 1023) / 1024);
    if ((long long)chunks * maps > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
    (void)hipGetLastError();
    if (d->dtype == SCAN2D_BF16)
        hipLaunchKernelGGL(scan2d_skip_step_kernel<bf16_t>, dim3((unsigned)(chunks * maps)), dim3(256), 0, stream,
                           static_cast<const bf16_t*>(delta), mask, static_cast<bf16_t*>(out), HW, d->Dc, chunks,
                           minus_inf ? 0xff80u : 0u);
    else
        hipLaunchKernelGGL(scan2d_skip_step_kernel<float>, dim3((unsigned)(chunks * maps)), dim3(256), 0, stream,
                           static_cast<const float*>(delta), mask, static_cast<float*>(out), HW, d->Dc, chunks,
                           minus_inf ? 0xff800000u : 0u);
    return hipGetLastError() == hipSuccess ? SCAN2D_OK : SCAN2D_ERR_LAUNCH_FAILED;
}

int skip_grad_launch(const scan2d_desc* d, const uint8_t* mask, void* ddelta, hipStream_t stream) {
    const size_t HW = (size_t)d->H * d->W;
    const long long maps = (long long)d->Bt * d->Dc;
    const unsigned chunks = (unsigned)((HW + 1023) / 1024);
    if ((long long)chunks * maps > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
    (void)hipGetLastError();
    if (d->dtype == SCAN2D_BF16)
        hipLaunchKernelGGL(scan2d_skip_grad_kernel<bf16_t>, dim3((unsigned)(chunks * maps)), dim3(256), 0, stream, mask,
                           static_cast<bf16_t*>(ddelta), HW, d->Dc, chunks);
    else
        hipLaunchKernelGGL(scan2d_skip_grad_kernel<float>, dim3((unsigned)(chunks * maps)), dim3(256), 0, stream, mask,
                           static_cast<float*>(ddelta), HW, d->Dc, chunks);
    return hipGetLastError() == hipSuccess ? SCAN2D_OK : SCAN2D_ERR_LAUNCH_FAILED;
}

int transpose_launch(int elem_bytes, const void* src, void* dst, long long planes, int H, int W, hipStream_t stream) {
    const unsigned tw = (unsigned)((W + 31) / 32), th = (unsigned)((H + 31) / 32);
    const long long blocks = planes * tw * th;
    if (blocks > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
    (void)hipGetLastError();
    if (elem_bytes == 4)
        hipLaunchKernelGGL(scan2d_transpose_kernel<uint32_t>, dim3((unsigned)blocks), dim3(256), 0, stream,
                           static_cast<const uint32_t*>(src), static_cast<uint32_t*>(dst), H, W, tw, th);
    else if (elem_bytes == 2)
        hipLaunchKernelGGL(scan2d_transpose_kernel<uint16_t>, dim3((unsigned)blocks), dim3(256), 0, stream,
                           static_cast<const uint16_t*>(src), static_cast<uint16_t*>(dst), H, W, tw, th);
    else
        hipLaunchKernelGGL(scan2d_transpose_kernel<uint8_t>, dim3((unsigned)blocks), dim3(256), 0, stream,
                           static_cast<const uint8_t*>(src), static_cast<uint8_t*>(dst), H, W, tw, th);
    return hipGetLastError() == hipSuccess ? SCAN2D_OK : SCAN2D_ERR_LAUNCH_FAILED;
}

namespace {
// Padding token: out = mask ? pad[c] : x (pad rounded to the storage type), one workgroup per map.
template <typename T>
__global__ __launch_bounds__(256) void scan2d_pad_fill_kernel(const T* __restrict__ x, const uint8_t* __restrict__ mask,
                                                              const float* __restrict__ pad, T* __restrict__ out, size_t HW, int Dc) {
    const size_t map = blockIdx.x;
    const uint32_t pbits = to_elem_bits<T>(pad[map % Dc]);
    const T* src = x + map * HW;
    T* dst = out + map * HW;
    const uint8_t* m = mask + (map / Dc) * HW;
    for (size_t e = threadIdx.x; e < HW; e += 256) {
        const uint32_t v = m[e] != 0 ? pbits : elem_bits(src + e);
        if constexpr (Elem<T>::kBytes == 4) reinterpret_cast<uint32_t*>(dst)[e] = v;
        else dst[e].bits = (uint16_t)v;
    }
}

// Gradient of the padding token: per map, the sum of dx over the masked cells (fixed order: strided partial sums
// per thread, then a tree over the workgroup) goes to ppad[map]; dx under the mask becomes +0.
template <typename T>
__global__ __launch_bounds__(256) void scan2d_pad_grad_kernel(T* __restrict__ dx, const uint8_t* __restrict__ mask,
                                                              float* __restrict__ ppad, size_t HW, int Dc) {
    __shared__ float sh[256];
    const size_t map = blockIdx.x;
    T* g = dx + map * HW;
    const uint8_t* m = mask + (map / Dc) * HW;
    float acc = 0.0f;
    for (size_t e = threadIdx.x; e < HW; e += 256) {
        if (m[e] != 0) {
            if constexpr (Elem<T>::kBytes == 4) { acc += __uint_as_float(elem_bits(g + e)); reinterpret_cast<uint32_t*>(g)[e] = 0u; }
            else { acc += __uint_as_float(elem_bits(g + e) << 16); g[e].bits = 0; }
        }
    }
    sh[threadIdx.x] = acc;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) sh[threadIdx.x] += sh[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) ppad[map] = sh[0];
}
// dpad[c] = sum over batch items of ppad[b][c] (all zeros when there is no mask: ppad == nullptr).
__global__ void scan2d_pad_batch_kernel(const float* __restrict__ ppad, float* __restrict__ dpad, int Bt, int Dc) {
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c < Dc) {
        float acc = 0.0f;
        if (ppad != nullptr)
            for (int b = 0; b < Bt; ++b) acc += ppad[(size_t)b * Dc + c];
        dpad[c] = acc;
    }
}
}  // namespace

int pad_fill_launch(const scan2d_desc* d, const void* x, const uint8_t* mask, const float* pad, void* out, hipStream_t stream) {
    const long long maps = (long long)d->Bt * d->Dc;
    if (maps > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
    const size_t HW = (size_t)d->H * d->W;
    (void)hipGetLastError();
    if (d->dtype == SCAN2D_BF16)
        hipLaunchKernelGGL(scan2d_pad_fill_kernel<bf16_t>, dim3((unsigned)maps), dim3(256), 0, stream, static_cast<const bf16_t*>(x), mask,
                           pad, static_cast<bf16_t*>(out), HW, d->Dc);
    else
        hipLaunchKernelGGL(scan2d_pad_fill_kernel<float>, dim3((unsigned)maps), dim3(256), 0, stream, static_cast<const float*>(x), mask,
                           pad, static_cast<float*>(out), HW, d->Dc);
    return hipGetLastError() == hipSuccess ? SCAN2D_OK : SCAN2D_ERR_LAUNCH_FAILED;
}

int pad_grad_launch(const scan2d_desc* d, const uint8_t* mask, void* dx, float* ppad, float* dpad, hipStream_t stream) {
    const long long maps = (long long)d->Bt * d->Dc;
    if (maps > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
    const size_t HW = (size_t)d->H * d->W;
    (void)hipGetLastError();
    if (mask != nullptr) {
        if (d->dtype == SCAN2D_BF16)
            hipLaunchKernelGGL(scan2d_pad_grad_kernel<bf16_t>, dim3((unsigned)maps), dim3(256), 0, stream, static_cast<bf16_t*>(dx), mask, ppad, HW, d->Dc);
        else
            hipLaunchKernelGGL(scan2d_pad_grad_kernel<float>, dim3((unsigned)maps), dim3(256), 0, stream, static_cast<float*>(dx), mask, ppad, HW, d->Dc);
    }
    hipLaunchKernelGGL(scan2d_pad_batch_kernel, dim3((d->Dc + 255) / 256), dim3(256), 0, stream,
                       mask != nullptr ? ppad : nullptr, dpad, d->Bt, d->Dc);
    return hipGetLastError() == hipSuccess ? SCAN2D_OK : SCAN2D_ERR_LAUNCH_FAILED;
}

}  // namespace scan2d
