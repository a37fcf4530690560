/* Driver for the sanitizer build of the CPU oracle (tests/test_oracle_sanitizers.py compiles this file together with
 * oracle/scan2d_oracle.c and oracle/scan2d_oracle_variants.c under -fsanitize=address,undefined and runs it): every
 * oracle entry point once on small inputs of every storage type, with and without the optional arguments.  Values do
 * not matter here (the pins check them); out-of-bounds accesses, leaks and undefined behaviour do. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_scan2d_fwd(int, int, int, int, int, int, const void*, const void*, const float*, const void*, const void*,
                      const float*, const uint8_t*, void*, int);
int oracle_scan2d_bwd(int, int, int, int, int, int, const void*, const void*, const float*, const void*, const void*,
                      const float*, const uint8_t*, const void*, void*, void*, float*, float*, float*, float*, int);
int oracle_scan2d_fwd_variants(int, int, int, int, int, int, const void*, const void*, const float*, const float*,
                               const void*, const void*, const float*, const uint8_t*, const float*, void*);
int oracle_scan2d_bwd_variants(int, int, int, int, int, int, const void*, const void*, const float*, const float*,
                               const void*, const void*, const float*, const uint8_t*, const float*, const void*,
                               void*, void*, float*, float*, float*, float*, float*, float*);
void oracle_round_to_bf16(const double*, uint16_t*, size_t);

static uint32_t state = 12345u;
static double rnd(void) { state = state * 1664525u + 1013904223u; return (double)(state >> 8) / 16777216.0; }

static void* fill(size_t n, int dtype, double lo, double hi) {
    const size_t eb = dtype == 0 ? 4 : (dtype == 1 ? 2 : 8);
    void* p = malloc(n * eb);
    size_t k;
    if (!p) exit(2);
    for (k = 0; k < n; ++k) {
        const double v = lo + (hi - lo) * rnd();
        if (dtype == 0) ((float*)p)[k] = (float)v;
        else if (dtype == 2) ((double*)p)[k] = v;
        else oracle_round_to_bf16(&v, (uint16_t*)p + k, 1);
    }
    return p;
}

int main(void) {
    const int shapes[4][5] = {{1, 1, 1, 1, 1}, {2, 3, 5, 7, 4}, {1, 2, 1, 9, 3}, {3, 1, 6, 1, 2}};   /* Bt, Dc, H, W, N */
    int s, dtype, opt, rc = 0;
    for (s = 0; s < 4; ++s)
        for (dtype = 0; dtype < 3; ++dtype)
            for (opt = 0; opt < 2; ++opt) {
                const int Bt = shapes[s][0], Dc = shapes[s][1], H = shapes[s][2], W = shapes[s][3], N = shapes[s][4];
                const size_t M = (size_t)Bt * Dc * H * W, S = (size_t)Bt * N * H * W, eb = dtype == 0 ? 4 : (dtype == 1 ? 2 : 8);
                void *x = fill(M, dtype, -1, 1), *dl = fill(M, dtype, 0.01, 0.5), *dy = fill(M, dtype, -1, 1);
                void *Bm = fill(S, dtype, -1, 1), *Cm = fill(S, dtype, -1, 1);
                float *A = fill((size_t)Dc * N, 0, -2, -0.1), *Av = fill((size_t)Dc * N, 0, -2, -0.1);
                float *D = fill((size_t)Dc, 0, -1, 1), *pad = fill((size_t)Dc, 0, -1, 1);
                uint8_t* mask = malloc((size_t)Bt * H * W);
                void *y = malloc(M * eb), *dx = malloc(M * eb), *dd = malloc(M * eb);
                float *dA = malloc((size_t)Dc * N * 4), *dAv = malloc((size_t)Dc * N * 4), *dB = malloc(S * 4), *dC = malloc(S * 4);
                float *dD = malloc((size_t)Dc * 4), *dP = malloc((size_t)Dc * 4);
                size_t k;
                if (!mask || !y || !dx || !dd || !dA || !dAv || !dB || !dC || !dD || !dP) return 2;
                for (k = 0; k < (size_t)Bt * H * W; ++k) mask[k] = rnd() < 0.3;
                rc |= oracle_scan2d_fwd(Bt, Dc, H, W, N, dtype, x, dl, A, Bm, Cm, opt ? D : NULL, opt ? mask : NULL, y, 1 + opt);
                rc |= oracle_scan2d_bwd(Bt, Dc, H, W, N, dtype, x, dl, A, Bm, Cm, opt ? D : NULL, opt ? mask : NULL, dy, dx, dd, dA, dB, dC,
                                        opt ? dD : NULL, 1 + opt);
                rc |= oracle_scan2d_fwd_variants(Bt, Dc, H, W, N, dtype, x, dl, A, opt ? Av : NULL, Bm, Cm, opt ? D : NULL, mask,
                                                 opt ? pad : NULL, y);
                rc |= oracle_scan2d_bwd_variants(Bt, Dc, H, W, N, dtype, x, dl, A, opt ? Av : NULL, Bm, Cm, opt ? D : NULL, mask,
                                                 opt ? pad : NULL, dy, dx, dd, dA, opt ? dAv : NULL, dB, dC, opt ? dD : NULL, opt ? dP : NULL);
                free(x); free(dl); free(dy); free(Bm); free(Cm); free(A); free(Av); free(D); free(pad); free(mask);
                free(y); free(dx); free(dd); free(dA); free(dAv); free(dB); free(dC); free(dD); free(dP);
            }
    /* argument errors must be reported, not crash */
    if (oracle_scan2d_fwd(0, 1, 1, 1, 1, 0, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, 1) != -1) rc |= 4;
    if (oracle_scan2d_fwd_variants(1, 1, 1, 1, 1, 7, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL) != -1) rc |= 4;
    printf(rc == 0 ? "sanitizer driver: ok\n" : "sanitizer driver: FAILED (%d)\n", rc);
    return rc;
}
