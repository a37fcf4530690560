/*
 * CPU oracle for the 2D selective scan (2DMamba, Sec. 3.3, Eq. 3, Eq. 5, Eq. 6 and the
 * output rule below Eq. 7; supplementary algorithm "2D selective scan").
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the plain definition written out as loops, in
 * double precision, with no blocking, fusion or re-association.  It shares no code,
 * header, table or helper with the GPU library and must never be called from the
 * product path.  Only tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * Layouts (dense, row-major, last index fastest):
 *   x, delta, y, dy, dx, ddelta : [Bt][Dc][H][W]   fp32, bf16 stored as uint16, or double
 *   Bm, Cm                      : [Bt][N][H][W]    same storage type as x
 *   dBm, dCm                    : [Bt][N][H][W]    fp32
 *   A, dA                       : [Dc][N]          fp32
 *   Dskip, dDskip               : [Dc]             fp32 (Dskip may be NULL: no skip term)
 *   mask                        : [Bt][H][W]       uint8, nonzero = background (may be NULL)
 *
 * Forward, for every batch item b, channel c and state n independently:
 *   x_eff[i,j] = mask[b,i,j] ? 0 : x[b,c,i,j]                 zero-token reading of Eq. 4
 *   a[i,j]     = exp(delta[b,c,i,j] * A[c,n])                 Eq. 3
 *   u[i,j]     = delta[b,c,i,j] * Bm[b,n,i,j] * x_eff[i,j]    Eq. 3 (B-bar = delta * B)
 *   hhor[i,j]  = a[i,j] * hhor[i,j-1] + u[i,j]                Eq. 5, hhor[i,-1] = 0
 *   h[i,j]     = a[i,j] * h[i-1,j]   + hhor[i,j]              Eq. 6, h[-1,j]   = 0
 *   y[b,c,i,j] = sum_n Cm[b,n,i,j] * h_n[i,j] + Dskip[c] * x_eff[i,j]
 *
 * Backward (the paper only states its structure: two forward scans rebuild the states,
 * a reverse vertical and a reverse horizontal scan carry the gradients, Supp. B).  The
 * formulas are the derivatives of the forward definition above:
 *   g[i,j]  = dy[i,j] * Cm[n,i,j] + a[i+1,j] * g[i+1,j]       dL/dh,     g[H,j] = 0
 *   q[i,j]  = g[i,j]              + a[i,j+1] * q[i,j+1]       dL/dhhor,  q[i,W] = 0
 *   da[i,j] = g[i,j] * h[i-1,j] + q[i,j] * hhor[i,j-1]
 *   ddelta  = sum_n ( da * a * A[c,n] + q * Bm * x_eff )
 *   dA[c,n] = sum_{b,i,j} da * a * delta
 *   dBm     = sum_c q * delta * x_eff
 *   dCm     = sum_c dy * h
 *   dx      = mask ? 0 : sum_n q * delta * Bm + Dskip[c] * dy
 *   dDskip  = sum_{b,i,j} dy * x_eff
 * Gradients are with respect to the arrays as passed (delta after softplus, A itself).
 *
 * Parity status: forward and backward are both pinned by the CPU test-suite (printed 3x3
 * exponents of Eq. 8, brute-force path-product form of Eq. 7, H=1 / W=1 reduction to the 1D
 * recurrence of Eq. 1-2, summed-area table for a == 1, separable matmul form for constant a,
 * finite differences and the adjoint identity for the backward).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ORACLE_F64 stores x, delta, Bm, Cm, y, dy, dx, ddelta as double; it exists so that the pin
 * tests (finite differences, closed forms) are not limited by fp32 storage rounding. */
enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F64 = 2 };

/* bf16 -> double, exact: the 16 stored bits are the upper half of an IEEE fp32. */
static double widen_bf16(uint16_t bits) {
    uint32_t w = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/* double -> bf16 bits with ONE rounding (nearest, ties to even), sub-normals included.
 * Relies on the default floating-point environment (nearbyint = ties-to-even). */
static uint16_t round_to_bf16(double v) {
    float f;
    uint32_t w;
    if (isnan(v)) return 0x7fc0;
    if (isinf(v)) return v > 0 ? 0x7f80 : 0xff80;
    if (v == 0.0) return signbit(v) ? 0x8000 : 0x0000;
    {
        int e = ilogb(v);
        double quantum, r;
        if (e < -126) e = -126;          /* sub-normal range shares the quantum of 2^-126 */
        quantum = ldexp(1.0, e - 7);     /* bf16 keeps 8 significant bits */
        r = nearbyint(v / quantum) * quantum;
        if (fabs(r) >= ldexp(1.0, 128)) return r > 0 ? 0x7f80 : 0xff80;
        f = (float)r;                    /* exact: r has at most 8 significant bits */
    }
    memcpy(&w, &f, sizeof w);
    return (uint16_t)(w >> 16);
}

static double load_elem(const void* p, int dtype, size_t idx) {
    if (dtype == ORACLE_BF16) return widen_bf16(((const uint16_t*)p)[idx]);
    if (dtype == ORACLE_F64) return ((const double*)p)[idx];
    return (double)((const float*)p)[idx];
}

static void store_elem(void* p, int dtype, size_t idx, double v) {
    if (dtype == ORACLE_BF16) ((uint16_t*)p)[idx] = round_to_bf16(v);
    else if (dtype == ORACLE_F64) ((double*)p)[idx] = v;
    else ((float*)p)[idx] = (float)v;
}

static int bad_args(int Bt, int Dc, int H, int W, int N, int dtype) {
    if (Bt < 1 || Dc < 1 || H < 1 || W < 1 || N < 1) return 1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16 && dtype != ORACLE_F64) return 1;
    return 0;
}

/* Forward.  Returns 0, or -1 on bad arguments / allocation failure.
 * threads <= 0 means "all cores"; maps (b,c) are independent, so they are the parallel loop. */
int oracle_scan2d_fwd(int Bt, int Dc, int H, int W, int N, int dtype,
                      const void* x, const void* delta, const float* A,
                      const void* Bm, const void* Cm, const float* Dskip,
                      const uint8_t* mask, void* y, int threads)
{
    const size_t HW = (size_t)H * (size_t)W;
    const long maps = (long)Bt * (long)Dc;
    int failed = 0;
    long m;
    if (bad_args(Bt, Dc, H, W, N, dtype) || !x || !delta || !A || !Bm || !Cm || !y) return -1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
    else omp_set_num_threads(omp_get_num_procs());
#else
    (void)threads;
#endif

#pragma omp parallel for schedule(dynamic, 1)
    for (m = 0; m < maps; ++m) {
        const int b = (int)(m / Dc), c = (int)(m % Dc);
        const size_t xoff = (size_t)m * HW;
        double* yacc = (double*)calloc(HW, sizeof(double));   /* sum over states */
        double* hrow = (double*)malloc((size_t)W * sizeof(double)); /* h of the row above */
        int n, i, j;
        if (!yacc || !hrow) {
            free(yacc); free(hrow);
#pragma omp atomic write
            failed = 1;
            continue;
        }
        for (n = 0; n < N; ++n) {
            const double An = (double)A[(size_t)c * N + n];
            const size_t soff = ((size_t)b * N + n) * HW;
            for (j = 0; j < W; ++j) hrow[j] = 0.0;            /* h[-1,j] = 0 */
            for (i = 0; i < H; ++i) {
                double hhor = 0.0;                            /* hhor[i,-1] = 0 */
                for (j = 0; j < W; ++j) {
                    const size_t p = (size_t)i * W + j;
                    const double dl = load_elem(delta, dtype, xoff + p);
                    const int bg = mask && mask[(size_t)b * HW + p];
                    const double xe = bg ? 0.0 : load_elem(x, dtype, xoff + p);
                    const double a = exp(dl * An);
                    const double u = dl * load_elem(Bm, dtype, soff + p) * xe;
                    double h;
                    hhor = a * hhor + u;                      /* Eq. 5 */
                    h = a * hrow[j] + hhor;                   /* Eq. 6 */
                    hrow[j] = h;
                    yacc[p] += load_elem(Cm, dtype, soff + p) * h;
                }
            }
        }
        for (i = 0; i < H; ++i) {
            for (j = 0; j < W; ++j) {
                const size_t p = (size_t)i * W + j;
                double v = yacc[p];
                if (Dskip) {
                    const int bg = mask && mask[(size_t)b * HW + p];
                    const double xe = bg ? 0.0 : load_elem(x, dtype, xoff + p);
                    v += (double)Dskip[c] * xe;
                }
                store_elem(y, dtype, xoff + p, v);
            }
        }
        free(yacc);
        free(hrow);
    }
    return failed ? -1 : 0;
}

/* Backward.  All gradient outputs are overwritten.  dDskip may be NULL iff Dskip is NULL.
 * Sums over channels (dBm, dCm) are accumulated per thread in double and added up in thread
 * order; sums over batch and positions (dA, dDskip) are accumulated in double. */
int oracle_scan2d_bwd(int Bt, int Dc, int H, int W, int N, int dtype,
                      const void* x, const void* delta, const float* A,
                      const void* Bm, const void* Cm, const float* Dskip,
                      const uint8_t* mask, const void* dy,
                      void* dx, void* ddelta, float* dA, float* dBm, float* dCm,
                      float* dDskip, int threads)
{
    const size_t HW = (size_t)H * (size_t)W;
    const size_t NHW = (size_t)N * HW;
    int nthr = 1, failed = 0, b, t;
    double *dA_acc = NULL, *dD_acc = NULL, *part = NULL;
    size_t k;
    if (bad_args(Bt, Dc, H, W, N, dtype) || !x || !delta || !A || !Bm || !Cm || !dy ||
        !dx || !ddelta || !dA || !dBm || !dCm) return -1;
    if ((Dskip != NULL) != (dDskip != NULL)) return -1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
    else omp_set_num_threads(omp_get_num_procs());
    nthr = threads > 0 ? threads : omp_get_num_procs();
#else
    (void)threads;
#endif
    dA_acc = (double*)calloc((size_t)Dc * N, sizeof(double));
    dD_acc = (double*)calloc((size_t)Dc, sizeof(double));
    part = (double*)malloc((size_t)nthr * 2 * NHW * sizeof(double)); /* per-thread dBm|dCm */
    if (!dA_acc || !dD_acc || !part) { free(dA_acc); free(dD_acc); free(part); return -1; }

    for (b = 0; b < Bt; ++b) {
        int c;
        memset(part, 0, (size_t)nthr * 2 * NHW * sizeof(double));
#pragma omp parallel for schedule(static) num_threads(nthr)
        for (c = 0; c < Dc; ++c) {
#ifdef _OPENMP
            const int tid = omp_get_thread_num();
#else
            const int tid = 0;
#endif
            double* pB = part + (size_t)tid * 2 * NHW;
            double* pC = pB + NHW;
            const size_t xoff = ((size_t)b * Dc + c) * HW;
            double* a    = (double*)malloc(HW * sizeof(double));
            double* hhor = (double*)malloc(HW * sizeof(double));
            double* h    = (double*)malloc(HW * sizeof(double));
            double* g    = (double*)malloc(HW * sizeof(double));
            double* q    = (double*)malloc(HW * sizeof(double));
            double* dxa  = (double*)calloc(HW, sizeof(double));
            double* dda  = (double*)calloc(HW, sizeof(double));
            int n, i, j;
            if (!a || !hhor || !h || !g || !q || !dxa || !dda) {
                free(a); free(hhor); free(h); free(g); free(q); free(dxa); free(dda);
#pragma omp atomic write
                failed = 1;
                continue;
            }
            for (n = 0; n < N; ++n) {
                const double An = (double)A[(size_t)c * N + n];
                const size_t soff = ((size_t)b * N + n) * HW;
                double dAn = 0.0;
                /* scan 1 (horizontal) and scan 2 (vertical): rebuild the forward states */
                for (i = 0; i < H; ++i) {
                    for (j = 0; j < W; ++j) {
                        const size_t p = (size_t)i * W + j;
                        const double dl = load_elem(delta, dtype, xoff + p);
                        const int bg = mask && mask[(size_t)b * HW + p];
                        const double xe = bg ? 0.0 : load_elem(x, dtype, xoff + p);
                        const double u = dl * load_elem(Bm, dtype, soff + p) * xe;
                        a[p] = exp(dl * An);
                        hhor[p] = a[p] * (j > 0 ? hhor[p - 1] : 0.0) + u;
                    }
                }
                for (i = 0; i < H; ++i)
                    for (j = 0; j < W; ++j) {
                        const size_t p = (size_t)i * W + j;
                        h[p] = a[p] * (i > 0 ? h[p - W] : 0.0) + hhor[p];
                    }
                /* scan 3: reverse vertical */
                for (i = H - 1; i >= 0; --i)
                    for (j = 0; j < W; ++j) {
                        const size_t p = (size_t)i * W + j;
                        const double up = (i + 1 < H) ? a[p + W] * g[p + W] : 0.0;
                        g[p] = load_elem(dy, dtype, xoff + p) * load_elem(Cm, dtype, soff + p) + up;
                    }
                /* scan 4: reverse horizontal */
                for (i = 0; i < H; ++i)
                    for (j = W - 1; j >= 0; --j) {
                        const size_t p = (size_t)i * W + j;
                        const double rt = (j + 1 < W) ? a[p + 1] * q[p + 1] : 0.0;
                        q[p] = g[p] + rt;
                    }
                /* local gradients */
                for (i = 0; i < H; ++i)
                    for (j = 0; j < W; ++j) {
                        const size_t p = (size_t)i * W + j;
                        const double dl = load_elem(delta, dtype, xoff + p);
                        const int bg = mask && mask[(size_t)b * HW + p];
                        const double xe = bg ? 0.0 : load_elem(x, dtype, xoff + p);
                        const double Bv = load_elem(Bm, dtype, soff + p);
                        const double da = g[p] * (i > 0 ? h[p - W] : 0.0)
                                        + q[p] * (j > 0 ? hhor[p - 1] : 0.0);
                        dda[p] += da * a[p] * An + q[p] * Bv * xe;
                        dAn    += da * a[p] * dl;
                        dxa[p] += q[p] * dl * Bv;
                        pB[(size_t)n * HW + p] += q[p] * dl * xe;
                        pC[(size_t)n * HW + p] += load_elem(dy, dtype, xoff + p) * h[p];
                    }
                dA_acc[(size_t)c * N + n] += dAn;
            }
            {
                double dD = 0.0;
                for (i = 0; i < H; ++i)
                    for (j = 0; j < W; ++j) {
                        const size_t p = (size_t)i * W + j;
                        const int bg = mask && mask[(size_t)b * HW + p];
                        const double dyv = load_elem(dy, dtype, xoff + p);
                        const double xe = bg ? 0.0 : load_elem(x, dtype, xoff + p);
                        double v = dxa[p];
                        if (Dskip) { v += (double)Dskip[c] * dyv; dD += dyv * xe; }
                        store_elem(dx, dtype, xoff + p, bg ? 0.0 : v);
                        store_elem(ddelta, dtype, xoff + p, dda[p]);
                    }
                dD_acc[c] += dD;
            }
            free(a); free(hhor); free(h); free(g); free(q); free(dxa); free(dda);
        }
        for (k = 0; k < NHW; ++k) {
            double sB = 0.0, sC = 0.0;
            for (t = 0; t < nthr; ++t) {
                sB += part[(size_t)t * 2 * NHW + k];
                sC += part[(size_t)t * 2 * NHW + NHW + k];
            }
            dBm[(size_t)b * NHW + k] = (float)sB;
            dCm[(size_t)b * NHW + k] = (float)sC;
        }
    }
    for (k = 0; k < (size_t)Dc * N; ++k) dA[k] = (float)dA_acc[k];
    if (dDskip) for (k = 0; k < (size_t)Dc; ++k) dDskip[k] = (float)dD_acc[k];
    free(dA_acc); free(dD_acc); free(part);
    return failed ? -1 : 0;
}

int oracle_num_procs(void)
{
#ifdef _OPENMP
    return omp_get_num_procs();
#else
    return 1;
#endif
}

/* Rounds n doubles to bf16 bits with the single nearest-even rounding used for every output of
 * the oracle (for the Python-level compositions around the two functions above). */
void oracle_round_to_bf16(const double* in, uint16_t* out, size_t n) {
    for (size_t k = 0; k < n; ++k) out[k] = round_to_bf16(in[k]);
}

