// Forward 2D selective scan for maps of at most 16 x 16 positions and 16 states when there are few of them (2DMamba
// Sec. 4.3 times 14 x 14 grids: the last stage of a hierarchical backbone).  Such a call is bound by the chain of
// dependent steps, not by work: a kernel that walks the rows one after the other pays H times the latency of a row
// step.  Here a workgroup of 256 threads owns one map and takes both recurrences as parallel scans:
//   1. thread (i, j) = (DPP row, lane) holds cell (i, j); Eq. 5 is a 16-lane DPP scan along j for all rows at once;
//   2. the row results pass through LDS, transposed, and thread (j, i) now holds cell (i, j); Eq. 6 is the same DPP
//      scan along i for all columns at once (the rows of a column are independent of the other columns);
//   3. y = sum over the states of C * h + Dskip * x, formed by the thread that holds the cell.
// Two scans of four DPP steps instead of H row steps.  Every global load is made in the first layout (a wavefront
// reads four row segments per instruction; the same cells read column-wise would touch sixteen cache lines per
// instruction, which made the texture path the bound); Cm, the step and x reach the second layout through LDS together
// with the row results, and the decay is recomputed there.  Cells past H or W lie to the right of / below every real
// cell, and both scans only run rightwards / downwards, so whatever they hold (valid memory is read: addresses are
// clamped) reaches no output.
#include "../../include/scan2d.h"
#include "scan2d_fwd.hpp"
#include "scan2d_variants.hpp"

namespace scan2d {
namespace {

constexpr int kTile = 16, kTilePitch = 17, kTileStates = 16;

__device__ __forceinline__ float tile_widen(float, uint32_t bits) { return __uint_as_float(bits); }
__device__ __forceinline__ float tile_widen(bf16_t, uint32_t bits) { return __uint_as_float(bits << 16); }

template <typename T, bool SP>
__global__ __launch_bounds__(256) void scan2d_fwd_tile16_kernel(const FwdArgs p) {
    // [value][column][row], value = row result of Eq. 5 per state, Cm per state, the step, x (0 under the mask)
    __shared__ float tr[(2 * kTileStates + 2) * kTile * kTilePitch];
    const int tid = threadIdx.x;
    const int r = tid >> 4, q = tid & 15;                  // DPP row and lane: (i, j) in step 1, (j, i) in step 2
    const long long map = blockIdx.x;
    const int H = p.H, W = p.W, N = p.N;
    const size_t HW = (size_t)H * W;
    const int b = (int)(map / p.Dc), c = (int)(map % p.Dc);
    const T* xm = reinterpret_cast<const T*>(p.x) + (size_t)map * HW;
    const T* dm = reinterpret_cast<const T*>(p.delta) + (size_t)map * HW;
    const uint8_t* mm = p.mask ? p.mask + (size_t)b * HW : nullptr;
    const T* Bb = reinterpret_cast<const T*>(p.Bm) + (size_t)b * N * HW;
    const T* Cb = reinterpret_cast<const T*>(p.Cm) + (size_t)b * N * HW;
    const uint32_t o1 = (uint32_t)(min(r, H - 1) * W + min(q, W - 1));   // this thread's cell in step 1, clamped into the map
    const bool live2 = q < H && r < W;                                   // its cell in step 2 is (q, r)

    // ---- everything this thread reads, requested at once
    uint32_t rB[kTileStates], rC[kTileStates];
    const uint32_t rx1 = elem_bits(xm + o1), rd1 = elem_bits(dm + o1), rm1 = mm ? (uint32_t)mm[o1] : 0u;
#pragma unroll
    for (int n = 0; n < kTileStates; ++n) {
        const size_t so = (size_t)min(n, N - 1) * HW;     // states past N re-read the last one and are not summed
        rB[n] = elem_bits(Bb + so + o1);
        rC[n] = elem_bits(Cb + so + o1);
    }
    float Ap[kTileStates];
#pragma unroll
    for (int n = 0; n < kTileStates; ++n) Ap[n] = p.A[(size_t)c * N + min(n, N - 1)] * kLog2e;
    const float dsk = p.Dskip != nullptr ? p.Dskip[c] : 0.0f;
    const float dbias = (SP && p.delta_bias != nullptr) ? p.delta_bias[c] : 0.0f;
    float* const put = tr + q * kTilePitch + r;            // step 1 writes [.][q][r]
    const float* const get = tr + r * kTilePitch + q;      // step 2 reads  [.][r][q]: the cell (q, r)
    constexpr int PLANE = kTile * kTilePitch;

    // ---- step 1: Eq. 5 along the lanes of every row
    {
        float dl = tile_widen(T{}, rd1);
        if constexpr (SP) dl = softplus_f32(dl + dbias);
        const float xe = rm1 != 0u ? 0.0f : tile_widen(T{}, rx1);
        const float dxe = dl * xe;
        put[2 * kTileStates * PLANE] = dl;
        put[(2 * kTileStates + 1) * PLANE] = xe;
#pragma unroll
        for (int n0 = 0; n0 < kTileStates; n0 += 4) {
            if (n0 < N) {                                  // uniform
                float P[4], Hh[4], cin[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    P[t] = __builtin_amdgcn_exp2f(dl * Ap[n0 + t]);
                    Hh[t] = dxe * tile_widen(T{}, rB[n0 + t]);
                    put[(kTileStates + n0 + t) * PLANE] = tile_widen(T{}, rC[n0 + t]);
                }
                group_scan<16, 4>(P, Hh, cin);
#pragma unroll
                for (int t = 0; t < 4; ++t) put[(n0 + t) * PLANE] = Hh[t];
            }
        }
    }
    __syncthreads();

    // ---- step 2: Eq. 6 along the lanes of every column, then the output rule
    const float dl = get[2 * kTileStates * PLANE];
    float yacc = dsk * get[(2 * kTileStates + 1) * PLANE];
#pragma unroll
    for (int n0 = 0; n0 < kTileStates; n0 += 4) {
        if (n0 < N) {
            float P[4], Hh[4], cin[4], Cv[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                P[t] = __builtin_amdgcn_exp2f(dl * Ap[n0 + t]);
                Hh[t] = get[(n0 + t) * PLANE];
                Cv[t] = get[(kTileStates + n0 + t) * PLANE];
            }
            group_scan<16, 4>(P, Hh, cin);
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (n0 + t < N) yacc = fmaf(Cv[t], Hh[t], yacc);
        }
    }
    if (live2) store_elem(reinterpret_cast<T*>(p.y) + (size_t)map * HW + (size_t)q * W + r, yacc);
}

}  // namespace

FwdKernel fwd_tile16_kernel(int dtype, bool sp) {
    if (dtype == SCAN2D_BF16) return sp ? scan2d_fwd_tile16_kernel<bf16_t, true> : scan2d_fwd_tile16_kernel<bf16_t, false>;
    return sp ? scan2d_fwd_tile16_kernel<float, true> : scan2d_fwd_tile16_kernel<float, false>;
}

}  // namespace scan2d
