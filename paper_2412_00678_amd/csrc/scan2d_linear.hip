// The linear layers of a 2DMamba block (Fig. 2: the projections into and out of the block's inner width; the design of
// the original block, Sec. 3.2) on channel-major maps:
//     out[b,o,p] = bias[o] + sum_c Wt[o,c] * in[b,c,p] (+ residual[b,o,p]),   p = position of the map,
// a GEMM with the positions as its wide dimension, on the matrix cores (v_mfma_f32_16x16x16_bf16 for bf16 storage,
// v_mfma_f32_16x16x4_f32 for fp32 storage, fp32 accumulation, one rounding after bias and residual).
//
// scan2d_linear_kernel: a workgroup of four wavefronts (2 x 2) owns a tile of 128 output channels x 128 positions and
// walks over the input channels 32 at a time.  Both operands pass through LDS, double-buffered, the next step's global
// loads in flight during the current step's products.  Wt is row-major in the contraction index, which is what an MFMA
// lane wants (4 consecutive channels of one row); `in` is channel-major, so a thread loads a 4 x 4 block (4 channels x
// 4 positions, one vector per channel), transposes it in registers and stores one vector per position: in LDS both
// operands are [row or position][channel] and every fragment is a single 64-bit (bf16) or 128-bit (fp32) read.  With
// fp32 storage the 16 channels of a group are contracted in the order (k-group of the lane, step), the same on both
// operands.  The output tile goes back through LDS as fp32 (the pipeline's buffers, in two halves for bf16) and leaves
// as whole rows of 128 positions with bias and residual added on the way.  Workgroups that share a tile of positions
// are mapped to the same XCD, so that the tile of `in` is read from HBM once.
// scan2d_linear_any_kernel: one thread per output, for maps whose H*W or channel count is not a multiple of 4.
#include "scan2d_block.hpp"

#include <algorithm>

#include "scan2d_common.hpp"

namespace scan2d {
namespace {

typedef short short4v __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) {       // nearest even, one v_cvt_pk_bf16_f32
    const float2v v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2v));
}

constexpr int kLinO = 128, kLinP = 128, kLinK = 32;
constexpr int kXcds = 8;
template <typename T> struct LinTile;
// row pitch in elements: the 16 lanes of a k-group read rows 80 B (bf16) / 144 B (fp32) apart, all banks distinct
template <> struct LinTile<bf16_t> { static constexpr int kPitch = kLinK + 8; };
template <> struct LinTile<float>  { static constexpr int kPitch = kLinK + 4; };
constexpr int kStagePitch = kLinP + 4;                                     // floats per staged output row

struct LinArgs {
    const void* in; const void* Wt; const float* bias; const void* res; void* out;
    int Cin, Cout, Bt, otiles;
    long long ptiles, P, total;     // tiles of positions per batch item, positions per map, workgroups with work
};

template <typename T>
__global__ __launch_bounds__(256) void scan2d_linear_kernel(const LinArgs p) {
    constexpr int EB = Elem<T>::kBytes, PITCH = LinTile<T>::kPitch;
    constexpr int OPERAND = kLinO * PITCH;                 // elements of one operand tile
    constexpr int ROUNDS = EB == 2 ? 2 : 1;                // the output tile is staged in this many parts
    using Raw = std::conditional_t<EB == 2, uint16_t, uint32_t>;
    using Vec = std::conditional_t<EB == 2, uint2, uint4>;
    extern __shared__ __align__(16) unsigned char smem[];
    Raw* const lds = reinterpret_cast<Raw*>(smem);         // [2 buffers][Wt tile, in tile][128][PITCH]
    float* const stage = reinterpret_cast<float*>(smem);   // [128 / ROUNDS][kStagePitch] after the products

    // workgroups that differ only in the tile of output channels follow each other on one XCD
    const long long per = (p.total + kXcds - 1) / kXcds;
    const long long wg = (long long)(blockIdx.x % kXcds) * per + blockIdx.x / kXcds;
    if (wg >= p.total) return;
    const int ot = (int)(wg % p.otiles);
    const long long rest = wg / p.otiles;
    const long long pt = rest % p.ptiles;
    const int b = (int)(rest / p.ptiles);
    const int o0 = ot * kLinO;
    const long long p0 = pt * kLinP;

    const int tid = threadIdx.x, l = tid & 63, wv = tid >> 6, g = l >> 4, n = l & 15;
    const int wo = wv >> 1, wp = wv & 1;
    const int Cin = p.Cin, Cout = p.Cout;
    const long long P = p.P;
    const T* Wt = static_cast<const T*>(p.Wt);
    const T* in = static_cast<const T*>(p.in) + (size_t)b * Cin * P;

    // ---- staging roles
    // Wt: vector v = tid + 256 * it covers row v / 8, channels 4 * (v % 8)..
    // in: 4 x 4 block: channels 4 * (tid / 32).., positions 4 * (tid % 32)..
    const int xc4 = tid >> 5, xp4 = tid & 31;
    const long long xpos = p0 + 4 * xp4;
    const bool xin = xpos < P;
    const T* xsrc = in + (size_t)min(xpos, P - 4);
    Vec wreg[4], xreg[4];
    auto load_global = [&](int k0) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int v = tid + 256 * it, o = o0 + (v >> 3), c = k0 + 4 * (v & 7);
            const Vec t = *reinterpret_cast<const Vec*>(Wt + (size_t)min(o, Cout - 1) * Cin + min(c, Cin - 4));
            wreg[it] = (o < Cout && c < Cin) ? t : Vec{};
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = k0 + 4 * xc4 + j;
            const Vec t = *reinterpret_cast<const Vec*>(xsrc + (size_t)min(c, Cin - 1) * P);
            xreg[j] = (xin && c < Cin) ? t : Vec{};
        }
    };
    auto store_lds = [&](int buf) {
        Raw* const wL = lds + (size_t)buf * 2 * OPERAND;
        Raw* const xL = wL + OPERAND;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int v = tid + 256 * it;
            *reinterpret_cast<Vec*>(wL + (size_t)(v >> 3) * PITCH + 4 * (v & 7)) = wreg[it];
        }
        Raw* const dst = xL + (size_t)(4 * xp4) * PITCH + 4 * xc4;
        if constexpr (EB == 2) {                           // xreg[j] = positions 0..3 of channel j, 16 bits each
            uint2 t0, t1, t2, t3;
            t0.x = (xreg[0].x & 0xffffu) | (xreg[1].x << 16);        t0.y = (xreg[2].x & 0xffffu) | (xreg[3].x << 16);
            t1.x = (xreg[0].x >> 16) | (xreg[1].x & 0xffff0000u);    t1.y = (xreg[2].x >> 16) | (xreg[3].x & 0xffff0000u);
            t2.x = (xreg[0].y & 0xffffu) | (xreg[1].y << 16);        t2.y = (xreg[2].y & 0xffffu) | (xreg[3].y << 16);
            t3.x = (xreg[0].y >> 16) | (xreg[1].y & 0xffff0000u);    t3.y = (xreg[2].y >> 16) | (xreg[3].y & 0xffff0000u);
            *reinterpret_cast<uint2*>(dst) = t0;
            *reinterpret_cast<uint2*>(dst + PITCH) = t1;
            *reinterpret_cast<uint2*>(dst + 2 * PITCH) = t2;
            *reinterpret_cast<uint2*>(dst + 3 * PITCH) = t3;
        } else {
            *reinterpret_cast<uint4*>(dst) = make_uint4(xreg[0].x, xreg[1].x, xreg[2].x, xreg[3].x);
            *reinterpret_cast<uint4*>(dst + PITCH) = make_uint4(xreg[0].y, xreg[1].y, xreg[2].y, xreg[3].y);
            *reinterpret_cast<uint4*>(dst + 2 * PITCH) = make_uint4(xreg[0].z, xreg[1].z, xreg[2].z, xreg[3].z);
            *reinterpret_cast<uint4*>(dst + 3 * PITCH) = make_uint4(xreg[0].w, xreg[1].w, xreg[2].w, xreg[3].w);
        }
    };

    float4v acc[4][4];                                     // [row block][column block] of this wavefront's 64 x 64
#pragma unroll
    for (int rb = 0; rb < 4; ++rb)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) acc[rb][cb] = float4v{0.0f, 0.0f, 0.0f, 0.0f};

    const int nk = (Cin + kLinK - 1) / kLinK;
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) load_global((kt + 1) * kLinK);
        const Raw* const wL = lds + (size_t)(kt & 1) * 2 * OPERAND + (size_t)(wo * 64 + n) * PITCH + 4 * g;
        const Raw* const xL = lds + (size_t)(kt & 1) * 2 * OPERAND + OPERAND + (size_t)(wp * 64 + n) * PITCH + 4 * g;
#pragma unroll
        for (int kg = 0; kg < kLinK / 16; ++kg) {
            if constexpr (EB == 2) {
                short4v af[4], bf[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const uint2 ta = *reinterpret_cast<const uint2*>(wL + (size_t)r * 16 * PITCH + kg * 16);
                    const uint2 tb = *reinterpret_cast<const uint2*>(xL + (size_t)r * 16 * PITCH + kg * 16);
                    af[r].x = (short)(ta.x & 0xffffu); af[r].y = (short)(ta.x >> 16); af[r].z = (short)(ta.y & 0xffffu); af[r].w = (short)(ta.y >> 16);
                    bf[r].x = (short)(tb.x & 0xffffu); bf[r].y = (short)(tb.x >> 16); bf[r].z = (short)(tb.y & 0xffffu); bf[r].w = (short)(tb.y >> 16);
                }
#pragma unroll
                for (int rb = 0; rb < 4; ++rb)
#pragma unroll
                    for (int cb = 0; cb < 4; ++cb) acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(af[rb], bf[cb], acc[rb][cb], 0, 0, 0);
            } else {
                float4 af[4], bf[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    af[r] = *reinterpret_cast<const float4*>(wL + (size_t)r * 16 * PITCH + kg * 16);
                    bf[r] = *reinterpret_cast<const float4*>(xL + (size_t)r * 16 * PITCH + kg * 16);
                }
#pragma unroll
                for (int rb = 0; rb < 4; ++rb)
#pragma unroll
                    for (int cb = 0; cb < 4; ++cb) {
                        acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[rb].x, bf[cb].x, acc[rb][cb], 0, 0, 0);
                        acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[rb].y, bf[cb].y, acc[rb][cb], 0, 0, 0);
                        acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[rb].z, bf[cb].z, acc[rb][cb], 0, 0, 0);
                        acc[rb][cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[rb].w, bf[cb].w, acc[rb][cb], 0, 0, 0);
                    }
            }
        }
        if (kt + 1 < nk) store_lds((kt + 1) & 1);
        __syncthreads();
    }

    // ---- the tile leaves through LDS: accumulator (rb, cb, r) of lane (n, g) is row wo*64 + rb*16 + 4g + r,
    // position wp*64 + cb*16 + n
    const T* res = p.res ? static_cast<const T*>(p.res) + (size_t)b * Cout * P : nullptr;
    T* out = static_cast<T*>(p.out) + (size_t)b * Cout * P;
    constexpr int ROWS = kLinO / ROUNDS;                   // rows per part: the rows of the wavefronts with wo == part
#pragma unroll
    for (int part = 0; part < ROUNDS; ++part) {
        if (ROUNDS == 1 || wo == part) {
            const int rbase = ROUNDS == 1 ? wo * 64 : 0;
#pragma unroll
            for (int rb = 0; rb < 4; ++rb)
#pragma unroll
                for (int cb = 0; cb < 4; ++cb)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        stage[(size_t)(rbase + rb * 16 + 4 * g + r) * kStagePitch + wp * 64 + cb * 16 + n] = acc[rb][cb][r];
        }
        __syncthreads();
        const int q = tid & 31, r0 = tid >> 5;             // 32 vectors per row, 8 rows per pass
        const long long pos = p0 + 4 * q;
#pragma unroll 4
        for (int it = 0; it < ROWS / 8; ++it) {
            const int row = r0 + 8 * it;
            const int o = o0 + part * ROWS + row;
            if (o < Cout && pos < P) {
                float4 v = *reinterpret_cast<const float4*>(stage + (size_t)row * kStagePitch + 4 * q);
                if (p.bias) { const float bv = p.bias[o]; v.x += bv; v.y += bv; v.z += bv; v.w += bv; }
                const size_t off = (size_t)o * P + pos;
                if constexpr (EB == 2) {
                    if (res) {
                        const uint2 rv = *reinterpret_cast<const uint2*>(res + off);
                        v.x += __uint_as_float(rv.x << 16); v.y += __uint_as_float(rv.x & 0xffff0000u);
                        v.z += __uint_as_float(rv.y << 16); v.w += __uint_as_float(rv.y & 0xffff0000u);
                    }
                    uint2 ov;
                    ov.x = pack2_bf16(v.x, v.y); ov.y = pack2_bf16(v.z, v.w);
                    *reinterpret_cast<uint2*>(out + off) = ov;
                } else {
                    if (res) {
                        const float4 rv = *reinterpret_cast<const float4*>(res + off);
                        v.x += rv.x; v.y += rv.y; v.z += rv.z; v.w += rv.w;
                    }
                    *reinterpret_cast<float4*>(out + off) = v;
                }
            }
        }
        if (part + 1 < ROUNDS) __syncthreads();
    }
}

// Any shape: one thread per output, channels in ascending order.
template <typename T>
__global__ __launch_bounds__(256) void scan2d_linear_any_kernel(const LinArgs p) {
    const long long P = p.P;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)p.Bt * p.Cout * P) return;
    const long long pos = idx % P;
    const int o = (int)((idx / P) % p.Cout), b = (int)(idx / (P * p.Cout));
    const T* in = static_cast<const T*>(p.in) + (size_t)b * p.Cin * P + pos;
    const T* w = static_cast<const T*>(p.Wt) + (size_t)o * p.Cin;
    auto widen = [](uint32_t bits) { return Elem<T>::kBytes == 4 ? __uint_as_float(bits) : __uint_as_float(bits << 16); };
    float acc = 0.0f;
    for (int c = 0; c < p.Cin; ++c) acc = fmaf(widen(elem_bits(w + c)), widen(elem_bits(in + (size_t)c * P)), acc);
    if (p.bias) acc += p.bias[o];
    if (p.res) acc += widen(elem_bits(static_cast<const T*>(p.res) + idx));
    store_elem(static_cast<T*>(p.out) + idx, acc);
}

template <typename T>
constexpr size_t linear_lds_bytes() { return (size_t)2 * 2 * kLinO * LinTile<T>::kPitch * Elem<T>::kBytes; }
static_assert(linear_lds_bytes<float>() >= (size_t)kLinO * kStagePitch * sizeof(float), "fp32: the whole output tile is staged");
static_assert(linear_lds_bytes<bf16_t>() >= (size_t)(kLinO / 2) * kStagePitch * sizeof(float), "bf16: half of the output tile is staged");

}  // namespace

bool allow_large_lds(const void* kernel, size_t bytes);   // scan2d_api.hip

int block_linear_launch(const scan2d_desc* d, int Cout, const void* in, const void* Wt, const float* bias, const void* residual,
                        void* out, hipStream_t stream) {
    if (Cout < 1) return SCAN2D_ERR_BAD_SHAPE;
    LinArgs a;
    a.in = in; a.Wt = Wt; a.bias = bias; a.res = residual; a.out = out;
    a.Cin = d->Dc; a.Cout = Cout; a.Bt = d->Bt;
    a.P = (long long)d->H * d->W;
    a.otiles = (Cout + kLinO - 1) / kLinO;
    a.ptiles = (a.P + kLinP - 1) / kLinP;
    a.total = (long long)a.otiles * a.ptiles * d->Bt;
    const bool bf16 = d->dtype == SCAN2D_BF16;
    (void)hipGetLastError();
    if (a.P % 4 == 0 && a.Cin % 4 == 0) {
        const long long grid = (a.total + kXcds - 1) / kXcds * kXcds;
        if (grid > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
        if (bf16) {
            hipLaunchKernelGGL(scan2d_linear_kernel<bf16_t>, dim3((unsigned)grid), dim3(256), linear_lds_bytes<bf16_t>(), stream, a);
        } else {
            if (!allow_large_lds(reinterpret_cast<const void*>(scan2d_linear_kernel<float>), linear_lds_bytes<float>())) return SCAN2D_ERR_LAUNCH_FAILED;
            hipLaunchKernelGGL(scan2d_linear_kernel<float>, dim3((unsigned)grid), dim3(256), linear_lds_bytes<float>(), stream, a);
        }
    } else {
        const long long blocks = ((long long)d->Bt * Cout * a.P + 255) / 256;
        if (blocks > 2147483647LL) return SCAN2D_ERR_BAD_SHAPE;
        if (bf16) hipLaunchKernelGGL(scan2d_linear_any_kernel<bf16_t>, dim3((unsigned)blocks), dim3(256), 0, stream, a);
        else hipLaunchKernelGGL(scan2d_linear_any_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, stream, a);
    }
    return hipGetLastError() == hipSuccess ? SCAN2D_OK : SCAN2D_ERR_LAUNCH_FAILED;
}

}  // namespace scan2d
