/*
 * CPU oracle for two variants of the 2D selective scan that 2DMamba ablates:
 *
 *   * the learnable padding token (Eq. 4 and the padding-token ablation table): a non-tissue (masked) cell
 *     holds a learnable value instead of a fixed zero.  At the level of the operator that is a per-channel
 *     value pad[c]:   x_eff[i,j] = mask[b,i,j] ? pad[c] : x[b,c,i,j];
 *   * an independent decay for the vertical scan (the supplement's ablation of re-using A-bar): the column
 *     recurrence uses its own parameter A_v[c,n]:   a_v[i,j] = exp(delta * A_v[c,n]),
 *     h[i,j] = a_v[i,j] * h[i-1,j] + hhor[i,j]       (the row recurrence keeps a = exp(delta * A)).
 *
 * THIS IS TEST INFRASTRUCTURE, written like scan2d_oracle.c: the definition as plain loops in double, no
 * blocking or re-association, nothing shared with the GPU library.  Layouts as there; pad and dpad are [Dc]
 * fp32, A_v and dA_v [Dc][N] fp32.  pad == NULL means the zero token, A_v == NULL means a_v = a: with both NULL
 * these functions compute exactly what oracle_scan2d_fwd / oracle_scan2d_bwd compute (a pin of the test-suite).
 *
 * Backward (derivatives of the definition; g = dL/dh, q = dL/dhhor as in scan2d_oracle.c):
 *   g[i,j]  = dy[i,j] * Cm[n,i,j] + a_v[i+1,j] * g[i+1,j]
 *   q[i,j]  = g[i,j]              + a[i,j+1]   * q[i,j+1]
 *   dah     = q[i,j] * hhor[i,j-1]          (through the row recurrence's a)
 *   dav     = g[i,j] * h[i-1,j]             (through the column recurrence's a_v)
 *   ddelta  = sum_n ( dah * a * A[c,n] + dav * a_v * A_v[c,n] + q * Bm * x_eff )
 *   dA[c,n] = sum dah * a * delta           dA_v[c,n] = sum dav * a_v * delta
 *   (without A_v: dA = sum (dah + dav) * a * delta, as in scan2d_oracle.c)
 *   dBm     = sum_c q * delta * x_eff       dCm = sum_c dy * h        dDskip = sum dy * x_eff
 *   dxfull  = sum_n q * delta * Bm + Dskip[c] * dy
 *   dx      = mask ? 0 : dxfull             dpad[c] = sum over b and the masked cells of dxfull
 *
 * Parity status: pinned by the CPU test-suite (central differences in every input including A_v and pad, the
 * reduction to the base oracle, closed forms for constant decays).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F64 = 2 };

static double widen_bf16v(uint16_t bits) {
    uint32_t w = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/* double -> bf16 bits, one rounding, nearest-even (default floating-point environment). */
static uint16_t round_to_bf16v(double v) {
    float f;
    uint32_t w;
    if (isnan(v)) return 0x7fc0;
    if (isinf(v)) return v > 0 ? 0x7f80 : 0xff80;
    if (v == 0.0) return signbit(v) ? 0x8000 : 0x0000;
    {
        int e = ilogb(v);
        double quantum, r;
        if (e < -126) e = -126;
        quantum = ldexp(1.0, e - 7);
        r = nearbyint(v / quantum) * quantum;
        if (fabs(r) >= ldexp(1.0, 128)) return r > 0 ? 0x7f80 : 0xff80;
        f = (float)r;
    }
    memcpy(&w, &f, sizeof w);
    return (uint16_t)(w >> 16);
}

static double ld(const void* p, int dtype, size_t idx) {
    if (dtype == ORACLE_BF16) return widen_bf16v(((const uint16_t*)p)[idx]);
    if (dtype == ORACLE_F64) return ((const double*)p)[idx];
    return (double)((const float*)p)[idx];
}

static void st(void* p, int dtype, size_t idx, double v) {
    if (dtype == ORACLE_BF16) ((uint16_t*)p)[idx] = round_to_bf16v(v);
    else if (dtype == ORACLE_F64) ((double*)p)[idx] = v;
    else ((float*)p)[idx] = (float)v;
}

static int bad(int Bt, int Dc, int H, int W, int N, int dtype) {
    if (Bt < 1 || Dc < 1 || H < 1 || W < 1 || N < 1) return 1;
    return dtype != ORACLE_F32 && dtype != ORACLE_BF16 && dtype != ORACLE_F64;
}

/* x_eff of one cell */
static double xeff(const void* x, int dtype, size_t idx, const uint8_t* mask, size_t midx, const float* pad, int c) {
    if (mask && mask[midx]) return pad ? (double)pad[c] : 0.0;
    return ld(x, dtype, idx);
}

int oracle_scan2d_fwd_variants(int Bt, int Dc, int H, int W, int N, int dtype,
                               const void* x, const void* delta, const float* A, const float* A_v,
                               const void* Bm, const void* Cm, const float* Dskip,
                               const uint8_t* mask, const float* pad, void* y)
{
    const size_t HW = (size_t)H * (size_t)W;
    double* yacc;
    double* hrow;
    int b, c, n, i, j;
    if (bad(Bt, Dc, H, W, N, dtype) || !x || !delta || !A || !Bm || !Cm || !y) return -1;
    yacc = (double*)malloc(HW * sizeof(double));
    hrow = (double*)malloc((size_t)W * sizeof(double));
    if (!yacc || !hrow) { free(yacc); free(hrow); return -1; }
    for (b = 0; b < Bt; ++b)
        for (c = 0; c < Dc; ++c) {
            const size_t xoff = ((size_t)b * Dc + c) * HW, moff = (size_t)b * HW;
            for (i = 0; i < (int)HW; ++i) yacc[i] = 0.0;
            for (n = 0; n < N; ++n) {
                const double An = (double)A[(size_t)c * N + n];
                const double Avn = A_v ? (double)A_v[(size_t)c * N + n] : An;
                const size_t soff = ((size_t)b * N + n) * HW;
                for (j = 0; j < W; ++j) hrow[j] = 0.0;                 /* h[-1,j] = 0 */
                for (i = 0; i < H; ++i) {
                    double hhor = 0.0;                                 /* hhor[i,-1] = 0 */
                    for (j = 0; j < W; ++j) {
                        const size_t p = (size_t)i * W + j;
                        const double dl = ld(delta, dtype, xoff + p);
                        const double xe = xeff(x, dtype, xoff + p, mask, moff + p, pad, c);
                        const double a = exp(dl * An), av = exp(dl * Avn);
                        hhor = a * hhor + dl * ld(Bm, dtype, soff + p) * xe;   /* row recurrence */
                        hrow[j] = av * hrow[j] + hhor;                         /* column recurrence, its own decay */
                        yacc[p] += ld(Cm, dtype, soff + p) * hrow[j];
                    }
                }
            }
            for (i = 0; i < (int)HW; ++i) {
                double v = yacc[i];
                if (Dskip) v += (double)Dskip[c] * xeff(x, dtype, xoff + i, mask, moff + i, pad, c);
                st(y, dtype, xoff + i, v);
            }
        }
    free(yacc);
    free(hrow);
    return 0;
}

/* dA_v must be non-NULL iff A_v is, dpad iff pad is, dDskip iff Dskip is. */
int oracle_scan2d_bwd_variants(int Bt, int Dc, int H, int W, int N, int dtype,
                               const void* x, const void* delta, const float* A, const float* A_v,
                               const void* Bm, const void* Cm, const float* Dskip,
                               const uint8_t* mask, const float* pad, const void* dy,
                               void* dx, void* ddelta, float* dA, float* dA_v, float* dBm, float* dCm,
                               float* dDskip, float* dpad)
{
    const size_t HW = (size_t)H * (size_t)W, NHW = (size_t)N * HW;
    double *a, *av, *hhor, *h, *g, *q, *dxa, *dda, *accB, *accC, *accA, *accAv, *accD, *accP;
    int b, c, n, i, j, rc = 0;
    size_t k;
    if (bad(Bt, Dc, H, W, N, dtype) || !x || !delta || !A || !Bm || !Cm || !dy || !dx || !ddelta || !dA || !dBm || !dCm)
        return -1;
    if ((Dskip != NULL) != (dDskip != NULL) || (A_v != NULL) != (dA_v != NULL) || (pad != NULL) != (dpad != NULL)) return -1;
    a = (double*)malloc(HW * sizeof(double));     av = (double*)malloc(HW * sizeof(double));
    hhor = (double*)malloc(HW * sizeof(double));  h = (double*)malloc(HW * sizeof(double));
    g = (double*)malloc(HW * sizeof(double));     q = (double*)malloc(HW * sizeof(double));
    dxa = (double*)malloc(HW * sizeof(double));   dda = (double*)malloc(HW * sizeof(double));
    accB = (double*)malloc(NHW * sizeof(double)); accC = (double*)malloc(NHW * sizeof(double));
    accA = (double*)calloc((size_t)Dc * N, sizeof(double));
    accAv = (double*)calloc((size_t)Dc * N, sizeof(double));
    accD = (double*)calloc((size_t)Dc, sizeof(double));
    accP = (double*)calloc((size_t)Dc, sizeof(double));
    if (!a || !av || !hhor || !h || !g || !q || !dxa || !dda || !accB || !accC || !accA || !accAv || !accD || !accP) rc = -1;
    for (b = 0; b < Bt && rc == 0; ++b) {
        const size_t moff = (size_t)b * HW;
        for (k = 0; k < NHW; ++k) { accB[k] = 0.0; accC[k] = 0.0; }
        for (c = 0; c < Dc; ++c) {
            const size_t xoff = ((size_t)b * Dc + c) * HW;
            for (k = 0; k < HW; ++k) { dxa[k] = 0.0; dda[k] = 0.0; }
            for (n = 0; n < N; ++n) {
                const double An = (double)A[(size_t)c * N + n];
                const double Avn = A_v ? (double)A_v[(size_t)c * N + n] : An;
                const size_t soff = ((size_t)b * N + n) * HW;
                /* the two forward scans */
                for (i = 0; i < H; ++i)
                    for (j = 0; j < W; ++j) {
                        const size_t p = (size_t)i * W + j;
                        const double dl = ld(delta, dtype, xoff + p);
                        const double xe = xeff(x, dtype, xoff + p, mask, moff + p, pad, c);
                        a[p] = exp(dl * An);
                        av[p] = exp(dl * Avn);
                        hhor[p] = a[p] * (j > 0 ? hhor[p - 1] : 0.0) + dl * ld(Bm, dtype, soff + p) * xe;
                        h[p] = av[p] * (i > 0 ? h[p - W] : 0.0) + hhor[p];
                    }
                /* reverse column scan, then reverse row scan */
                for (i = H - 1; i >= 0; --i)
                    for (j = 0; j < W; ++j) {
                        const size_t p = (size_t)i * W + j;
                        g[p] = ld(dy, dtype, xoff + p) * ld(Cm, dtype, soff + p) + (i + 1 < H ? av[p + W] * g[p + W] : 0.0);
                    }
                for (i = 0; i < H; ++i)
                    for (j = W - 1; j >= 0; --j) {
                        const size_t p = (size_t)i * W + j;
                        q[p] = g[p] + (j + 1 < W ? a[p + 1] * q[p + 1] : 0.0);
                    }
                /* local gradients */
                for (i = 0; i < H; ++i)
                    for (j = 0; j < W; ++j) {
                        const size_t p = (size_t)i * W + j;
                        const double dl = ld(delta, dtype, xoff + p);
                        const double xe = xeff(x, dtype, xoff + p, mask, moff + p, pad, c);
                        const double Bv = ld(Bm, dtype, soff + p);
                        const double dah = q[p] * (j > 0 ? hhor[p - 1] : 0.0);
                        const double dav = g[p] * (i > 0 ? h[p - W] : 0.0);
                        dda[p] += dah * a[p] * An + dav * av[p] * Avn + q[p] * Bv * xe;
                        accA[(size_t)c * N + n] += dah * a[p] * dl;
                        accAv[(size_t)c * N + n] += dav * av[p] * dl;
                        dxa[p] += q[p] * dl * Bv;
                        accB[(size_t)n * HW + p] += q[p] * dl * xe;
                        accC[(size_t)n * HW + p] += ld(dy, dtype, xoff + p) * h[p];
                    }
            }
            for (k = 0; k < HW; ++k) {
                const int bg = mask && mask[moff + k];
                const double dyv = ld(dy, dtype, xoff + k);
                double full = dxa[k];
                if (Dskip) {
                    full += (double)Dskip[c] * dyv;
                    accD[c] += dyv * xeff(x, dtype, xoff + k, mask, moff + k, pad, c);
                }
                if (bg) accP[c] += full;
                st(dx, dtype, xoff + k, bg ? 0.0 : full);
                st(ddelta, dtype, xoff + k, dda[k]);
            }
        }
        for (k = 0; k < NHW; ++k) { dBm[(size_t)b * NHW + k] = (float)accB[k]; dCm[(size_t)b * NHW + k] = (float)accC[k]; }
    }
    if (rc == 0) {
        for (k = 0; k < (size_t)Dc * N; ++k) {
            if (A_v) { dA[k] = (float)accA[k]; dA_v[k] = (float)accAv[k]; }
            else dA[k] = (float)(accA[k] + accAv[k]);          /* one parameter drives both decays */
        }
        for (k = 0; k < (size_t)Dc; ++k) {
            if (dDskip) dDskip[k] = (float)accD[k];
            if (dpad) dpad[k] = (float)accP[k];
        }
    }
    free(a); free(av); free(hhor); free(h); free(g); free(q); free(dxa); free(dda);
    free(accB); free(accC); free(accA); free(accAv); free(accD); free(accP);
    return rc;
}
