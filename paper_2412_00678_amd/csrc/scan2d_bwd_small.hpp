// Backward 2D selective scan for small maps (W <= 16, H <= 16, N <= 16): the 14x14 grids of
// the last stage of a hierarchical backbone (2DMamba Sec. 4.3), the four scans of Supp. B.
//
// One wavefront owns one map (batch item, channel).  Its four DPP rows split the states (NW per
// lane), lane l of a row owns column l.  A map this small fits the register file whole: the
// forward sweep (scans 1 and 2) leaves h[i-1,j] and hhor[i,j-1] of every row in registers, the
// reverse sweep (scans 3 and 4) walks back up.  No checkpoints, no bands, no LDS, no barrier.
// The sums over states (ddelta, dx) are finished inside the wave with two lane exchanges.  The
// sums over channels (dBm, dCm) are written per channel and added up by the reduction kernel
// that the general path uses too - for maps this small those partial sums are a few MB.
// Every access is a single element; the loads of the next PD rows are kept in flight.
#pragma once

#include "scan2d_bwd_kernels.hpp"
#include "scan2d_fwd_small.hpp"   // raw_to_float

namespace scan2d {

template <typename T, int NW, bool SP = false>
__global__ __launch_bounds__(256) void scan2d_bwd_small_kernel(const BwdArgs p) {
    constexpr int HM = 16;                                // most rows a map may have
    constexpr int PD = NW >= 4 ? 2 : 4;                   // rows of loads in flight
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l = lane & 15, g = lane >> 4;
    const long long maps = (long long)p.Bt * p.Dc;
    const long long map = (long long)blockIdx.x * 4 + wave;
    if (map >= maps) return;                              // uniform over the wave; the kernel has no barrier
    const int H = p.H, W = p.W, N = p.N;
    const size_t HW = (size_t)H * W;
    const int b = (int)(map / p.Dc), c = (int)(map % p.Dc);
    const int n0 = g * NW;
    const int nvalid = max(0, min(NW, N - n0));
    const bool in = l < W;
    const uint32_t lc = in ? (uint32_t)l : 0u;            // lanes past the map re-read column 0 and store nothing

    const T* xm = reinterpret_cast<const T*>(p.x) + (size_t)map * HW;
    const T* dm = reinterpret_cast<const T*>(p.delta) + (size_t)map * HW;
    const T* dym = reinterpret_cast<const T*>(p.dy) + (size_t)map * HW;
    T* dxm = reinterpret_cast<T*>(p.dx) + (size_t)map * HW;
    T* ddm = reinterpret_cast<T*>(p.ddelta) + (size_t)map * HW;
    const uint8_t* mm = p.mask ? p.mask + (size_t)b * HW : nullptr;
    // state planes of this batch item (inputs) and of this map (partial sums, CG = Dc: one per
    // channel); so[s] = element offset of the lane's s-th state, N*H*W <= 4096 here
    const T* Bb = reinterpret_cast<const T*>(p.Bm) + (size_t)b * N * HW;
    const T* Cb = reinterpret_cast<const T*>(p.Cm) + (size_t)b * N * HW;
    float* pBb = p.pB + ((size_t)b * p.CG + c) * N * HW;
    float* pCb = p.pC + ((size_t)b * p.CG + c) * N * HW;
    uint32_t so[NW];
    float An[NW], Ap[NW];
#pragma unroll
    for (int s = 0; s < NW; ++s) {
        const int n = min(n0 + s, N - 1);                 // states past N re-read the last one and store nothing
        so[s] = (uint32_t)n * (uint32_t)HW;
        An[s] = p.A[(size_t)c * N + n];
        Ap[s] = An[s] * kLog2e;
    }
    const float dsk = (g == 0 && p.Dskip != nullptr) ? p.Dskip[c] : 0.0f;
    const float dbias = (SP && p.delta_bias != nullptr) ? p.delta_bias[c] : 0.0f;   // SP: delta = softplus(raw + bias)

    // ---- scans 1 and 2, top to bottom: h[i-1,j] and hhor[i,j-1] of every row stay in registers
    float hprev[HM][NW], hhl[HM][NW];
    {
        uint32_t rx[PD], rd[PD], rm[PD], rB[PD][NW];
        auto request = [&](int slot, int i) {
            const size_t o = (size_t)i * W + lc;
            rx[slot] = elem_bits(xm + o);
            rd[slot] = elem_bits(dm + o);
            rm[slot] = mm ? (uint32_t)mm[o] : 0u;
#pragma unroll
            for (int s = 0; s < NW; ++s) rB[slot][s] = elem_bits(Bb + so[s] + o);
        };
#pragma unroll
        for (int r = 0; r < PD; ++r)
            if (r < H) request(r, r);
        float hcur[NW];
#pragma unroll
        for (int s = 0; s < NW; ++s) hcur[s] = 0.0f;
#pragma unroll
        for (int i = 0; i < HM; ++i) {
            if (i < H) {                                  // uniform
                const int slot = i % PD;               // a constant once the loop is unrolled
                float dl = raw_to_float(T{}, rd[slot]);
                if constexpr (SP) dl = softplus_f32(dl + dbias);
                const float xe = rm[slot] != 0u ? 0.0f : raw_to_float(T{}, rx[slot]);
                const float dxe = dl * xe;
                float P[NW], Hh[NW], cin[NW], a[NW];
#pragma unroll
                for (int s = 0; s < NW; ++s) {
                    a[s] = __builtin_amdgcn_exp2f(dl * Ap[s]);
                    P[s] = a[s];
                    Hh[s] = dxe * raw_to_float(T{}, rB[slot][s]);
                }
                if (i + PD < H) request(slot, i + PD);
                group_scan<16, NW>(P, Hh, cin);           // Hh = hhor[i,j], cin = hhor[i,j-1]
#pragma unroll
                for (int s = 0; s < NW; ++s) {
                    hhl[i][s] = cin[s];
                    hprev[i][s] = hcur[s];
                    hcur[s] = fmaf(a[s], hcur[s], Hh[s]);
                }
            }
        }
    }

    // ---- scans 3 and 4, bottom to top
    uint32_t rx[PD], rd[PD], ry[PD], rm[PD], rB[PD][NW], rC[PD][NW];
    auto request = [&](int slot, int i) {
        const size_t o = (size_t)i * W + lc;
        rx[slot] = elem_bits(xm + o);
        rd[slot] = elem_bits(dm + o);
        ry[slot] = elem_bits(dym + o);
        rm[slot] = mm ? (uint32_t)mm[o] : 0u;
#pragma unroll
        for (int s = 0; s < NW; ++s) {
            rB[slot][s] = elem_bits(Bb + so[s] + o);
            rC[slot][s] = elem_bits(Cb + so[s] + o);
        }
    };
#pragma unroll
    for (int r = 0; r < PD; ++r)
        if (H - 1 - r >= 0) request(r, H - 1 - r);
    float ga[NW], dAb[NW], dDb = 0.0f;
#pragma unroll
    for (int s = 0; s < NW; ++s) { ga[s] = 0.0f; dAb[s] = 0.0f; }     // g below the map is 0
#pragma unroll
    for (int k = 0; k < HM; ++k) {                        // k-th row from the bottom, i = H - 1 - k
        const int i = H - 1 - k;
        if (i >= 0) {                                     // uniform
            const int slot = k % PD;                   // a constant once the loop is unrolled
            const float traw = SP ? raw_to_float(T{}, rd[slot]) + dbias : raw_to_float(T{}, rd[slot]);
            const float dl = SP ? softplus_f32(traw) : traw;
            const bool masked = rm[slot] != 0u;
            const float xe = masked ? 0.0f : raw_to_float(T{}, rx[slot]);
            const float dyv = in ? raw_to_float(T{}, ry[slot]) : 0.0f;   // nothing flows out of a lane past the map
            const float dxe = dl * xe;
            float Bv[NW], Cv[NW];
#pragma unroll
            for (int s = 0; s < NW; ++s) {
                Bv[s] = raw_to_float(T{}, rB[slot][s]);
                Cv[s] = raw_to_float(T{}, rC[slot][s]);
            }
            if (i - PD >= 0) request(slot, i - PD);
            dDb = fmaf(dyv, xe, dDb);
            float a[NW], gq[NW], Pq[NW], Q[NW], qin[NW];
#pragma unroll
            for (int s = 0; s < NW; ++s) {
                a[s] = __builtin_amdgcn_exp2f(dl * Ap[s]);
                gq[s] = fmaf(dyv, Cv[s], ga[s]);          // scan 3: g[i,j]
                ga[s] = a[s] * gq[s];
                Pq[s] = from_right<16>(a[s]);             // a[i,j+1]
                Q[s] = gq[s];
            }
            float ar[NW];
#pragma unroll
            for (int s = 0; s < NW; ++s) ar[s] = Pq[s];
            group_scan_left<16, NW>(Pq, Q, qin);          // qin = q[i,j+1]
            float ddl = 0.0f, dxl = dsk * dyv;
            // index of the values of row i in the register arrays: i = H - 1 - k is not a compile-time
            // constant, so the arrays are read through a uniform switch over k-th-from-bottom rows
            float hp[NW], hl[NW];
#pragma unroll
            for (int r = 0; r < HM; ++r)
                if (r == i) {
#pragma unroll
                    for (int s = 0; s < NW; ++s) { hp[s] = hprev[r][s]; hl[s] = hhl[r][s]; }
                }
#pragma unroll
            for (int s = 0; s < NW; ++s) {
                const float q = fmaf(ar[s], qin[s], gq[s]);                 // scan 4: q[i,j]
                const float hh = fmaf(a[s], hl[s], dxe * Bv[s]);            // hhor[i,j]
                const float hv = fmaf(a[s], hp[s], hh);                     // h[i,j]
                const float da = fmaf(gq[s], hp[s], q * hl[s]);
                const float t = da * a[s];
                if (s < nvalid) {
                    dAb[s] = fmaf(t, dl, dAb[s]);
                    ddl = fmaf(t, An[s], fmaf(q * Bv[s], xe, ddl));
                    dxl = fmaf(q * dl, Bv[s], dxl);
                    if (in) {
                        pBb[so[s] + (uint32_t)(i * W + l)] = q * dxe;
                        pCb[so[s] + (uint32_t)(i * W + l)] = dyv * hv;
                    }
                }
            }
            // sums over the four lane groups: rows 0+1 and 2+3, then the two halves
            ddl += __shfl_xor(ddl, 16);
            ddl += __shfl_xor(ddl, 32);
            dxl += __shfl_xor(dxl, 16);
            dxl += __shfl_xor(dxl, 32);
            if (g == 0 && in) {
                store_elem(ddm + (size_t)i * W + l, SP ? ddl * logistic_f32(traw) : ddl);
                store_elem(dxm + (size_t)i * W + l, masked ? 0.0f : dxl);
            }
        }
    }

    // dA[b,c,n] and dDskip[b,c]: sums over the 16 lanes of the row in a fixed order
#pragma unroll
    for (int s = 0; s < NW; ++s) {
        const float v = row_sum16(in ? dAb[s] : 0.0f);
        if (l == 0 && s < nvalid) p.pA[((size_t)b * p.Dc + c) * N + n0 + s] = v;
    }
    const float vD = row_sum16(dDb);
    if (l == 0 && g == 0 && p.pD != nullptr) p.pD[(size_t)b * p.Dc + c] = vD;
}

}  // namespace scan2d
