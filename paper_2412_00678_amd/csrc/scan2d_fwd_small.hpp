// Forward 2D selective scan for narrow maps (W <= 32): the 14x14 to 28x28 grids of the last
// stages of a hierarchical backbone (2DMamba Sec. 4.3 times 14x14 and calls it typical).
//
// One wavefront owns one map.  Its four DPP rows split the N states (NW = ceil(N/4) per lane);
// lane l of a row owns the KS columns [l*KS, l*KS+KS), so a row of 16 lanes covers 16 or 32
// columns and 14 of 16 lanes work on a 14-wide map.  Eq. 5 is a 16-lane DPP scan per state,
// Eq. 6 one FMA on registers that persist from row to row, and the sum over states of
// y = C.h is finished inside the wave with two lane exchanges - no LDS, no barrier, so the
// short maps (a dozen rows) are not spent waiting at barriers.  Every access is a single
// element: any W and any row alignment is handled the same way.  The inputs of the next PD
// rows are always in flight (a ring of raw registers), because with so few rows per map it is
// the load latency per row, not the arithmetic, that sets the run time.
#pragma once

#include "scan2d_fwd.hpp"

namespace scan2d {

__device__ __forceinline__ float raw_to_float(float, uint32_t bits) { return __uint_as_float(bits); }
__device__ __forceinline__ float raw_to_float(bf16_t, uint32_t bits) { return __uint_as_float(bits << 16); }

template <typename T, int KS, int NW, int PD, bool SP = false>
__global__ __launch_bounds__(256) void scan2d_fwd_small_kernel(const FwdArgs p) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l = lane & 15, g = lane >> 4;
    const long long map = (long long)blockIdx.x * 4 + wave;
    if (map >= p.maps) return;                            // uniform over the wave; the kernel has no barrier
    const int H = p.H, W = p.W, N = p.N;
    const size_t HW = (size_t)H * W;
    const int b = (int)(map / p.Dc), c = (int)(map % p.Dc);
    const int n0 = g * NW;
    const int nvalid = max(0, min(NW, N - n0));           // states of this lane group that exist
    int col[KS];
    uint32_t lc[KS];
    bool in[KS];
#pragma unroll
    for (int k = 0; k < KS; ++k) { col[k] = l * KS + k; in[k] = col[k] < W; lc[k] = in[k] ? (uint32_t)col[k] : 0u; }

    const T* xm = reinterpret_cast<const T*>(p.x) + (size_t)map * HW;
    const T* dm = reinterpret_cast<const T*>(p.delta) + (size_t)map * HW;
    T* ym = reinterpret_cast<T*>(p.y) + (size_t)map * HW;
    const uint8_t* mm = p.mask ? p.mask + (size_t)b * HW : nullptr;
    const T* Bs[NW];
    const T* Cs[NW];
    float Ap[NW], h[NW][KS];
#pragma unroll
    for (int s = 0; s < NW; ++s) {
        const int n = min(n0 + s, N - 1);                 // states past N re-read the last one and are not summed
        Bs[s] = reinterpret_cast<const T*>(p.Bm) + ((size_t)b * N + n) * HW;
        Cs[s] = reinterpret_cast<const T*>(p.Cm) + ((size_t)b * N + n) * HW;
        Ap[s] = p.A[(size_t)c * N + n] * kLog2e;
#pragma unroll
        for (int k = 0; k < KS; ++k) h[s][k] = 0.0f;
    }
    const float dsk = (g == 0 && p.Dskip != nullptr) ? p.Dskip[c] : 0.0f;
    const float dbias = (SP && p.delta_bias != nullptr) ? p.delta_bias[c] : 0.0f;   // SP: delta = softplus(raw + bias)

    // ring of raw registers: row i waits in slot i % PD
    uint32_t rx[PD][KS], rd[PD][KS], rm[PD][KS], rB[PD][NW][KS], rC[PD][NW][KS];
    auto request = [&](int slot, int i) {
        const size_t ro = (size_t)i * W;
#pragma unroll
        for (int k = 0; k < KS; ++k) {
            rx[slot][k] = elem_bits(xm + ro + lc[k]);
            rd[slot][k] = elem_bits(dm + ro + lc[k]);
            rm[slot][k] = mm ? (uint32_t)mm[ro + lc[k]] : 0u;
        }
#pragma unroll
        for (int s = 0; s < NW; ++s)
#pragma unroll
            for (int k = 0; k < KS; ++k) {
                rB[slot][s][k] = elem_bits(Bs[s] + ro + lc[k]);
                rC[slot][s][k] = elem_bits(Cs[s] + ro + lc[k]);
            }
    };
#pragma unroll
    for (int r = 0; r < PD; ++r)
        if (r < H) request(r, r);

    for (int i0 = 0; i0 < H; i0 += PD) {
#pragma unroll
        for (int r = 0; r < PD; ++r) {
            const int i = i0 + r;
            if (i < H) {                                  // uniform
                float dl[KS], xe[KS], dxe[KS], yacc[KS], Bv[NW][KS], Cv[NW][KS];
#pragma unroll
                for (int k = 0; k < KS; ++k) {
                    dl[k] = raw_to_float(T{}, rd[r][k]);
                    if constexpr (SP) dl[k] = softplus_f32(dl[k] + dbias);
                    xe[k] = rm[r][k] != 0u ? 0.0f : raw_to_float(T{}, rx[r][k]);
                    dxe[k] = dl[k] * xe[k];
                    yacc[k] = dsk * xe[k];
                }
#pragma unroll
                for (int s = 0; s < NW; ++s)
#pragma unroll
                    for (int k = 0; k < KS; ++k) {
                        Bv[s][k] = raw_to_float(T{}, rB[r][s][k]);
                        Cv[s][k] = raw_to_float(T{}, rC[r][s][k]);
                    }
                if (i + PD < H) request(r, i + PD);

                constexpr int SC = NW >= 4 ? 4 : NW;      // states scanned together
#pragma unroll
                for (int s0 = 0; s0 < NW; s0 += SC) {
                    float a[SC][KS], hl[SC][KS], P[SC], Hh[SC], cin[SC];
#pragma unroll
                    for (int t = 0; t < SC; ++t) {
#pragma unroll
                        for (int k = 0; k < KS; ++k) a[t][k] = __builtin_amdgcn_exp2f(dl[k] * Ap[s0 + t]);
                        hl[t][0] = dxe[0] * Bv[s0 + t][0];
                        P[t] = a[t][0];
#pragma unroll
                        for (int k = 1; k < KS; ++k) {
                            hl[t][k] = fmaf(a[t][k], hl[t][k - 1], dxe[k] * Bv[s0 + t][k]);
                            P[t] *= a[t][k];
                        }
                        Hh[t] = hl[t][KS - 1];
                    }
                    group_scan<16, SC>(P, Hh, cin);
#pragma unroll
                    for (int t = 0; t < SC; ++t) {
                        float pl = 1.0f;
#pragma unroll
                        for (int k = 0; k < KS; ++k) {
                            pl *= a[t][k];
                            const float hh = (k == KS - 1) ? Hh[t] : fmaf(pl, cin[t], hl[t][k]);   // Eq. 5
                            h[s0 + t][k] = fmaf(a[t][k], h[s0 + t][k], hh);                        // Eq. 6
                            if (s0 + t < nvalid) yacc[k] = fmaf(Cv[s0 + t][k], h[s0 + t][k], yacc[k]);
                        }
                    }
                }
                // sum over the four lane groups: rows 0+1 and 2+3, then the two halves
#pragma unroll
                for (int k = 0; k < KS; ++k) {
                    float v = yacc[k];
                    v += __shfl_xor(v, 16);
                    v += __shfl_xor(v, 32);
                    if (g == 0 && in[k]) store_elem(ym + (size_t)i * W + col[k], v);
                }
            }
        }
    }
}

}  // namespace scan2d
