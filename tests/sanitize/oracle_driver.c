/* Drives oracle/mlpmoe_oracle.c under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only):
 * ragged sizes, empty and inactive branches, T = 0, d_inter = 0, both modes, the routed form and the
 * hidden-intermediate function.  Prints "ok" and exits 0; any sanitizer report aborts the run. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_mlpmoe_forward(const float *, const float *, const float *, const float *, const int32_t *, const float *,
                          const uint8_t *, int, int, int, int, int, double *);
int oracle_mlpmoe_forward_routed(const float *, const float *, const float *, const float *, const int32_t *,
                                 const float *, const uint8_t *, const uint8_t *, int, int, int, int, int, double *);
int oracle_mlpmoe_hidden(const float *, const float *, const float *, const int32_t *, const float *, const uint8_t *,
                         int, int, int, int, int, double *, double *, double *, double *, double *);
int oracle_dense_swiglu(const float *, const float *, const float *, const float *, int, int, int, double *);

static float *rnd(size_t n, unsigned *s)
{
    float *p = (float *)malloc(sizeof(float) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) {
        *s = *s * 1664525u + 1013904223u;
        p[i] = ((float)(*s >> 8) / 8388608.0f - 1.0f) * 0.5f;
    }
    return p;
}

static int run_case(int T, int d_model, const int32_t *off, const uint8_t *mask, int B)
{
    unsigned seed = 12345u + (unsigned)(T * 31 + d_model);
    const int d_inter = off[B];
    float *x = rnd((size_t)T * d_model, &seed), *Wg = rnd((size_t)d_inter * d_model, &seed);
    float *Wu = rnd((size_t)d_inter * d_model, &seed), *Wd = rnd((size_t)d_model * d_inter, &seed);
    float *alpha = rnd((size_t)B, &seed);
    uint8_t *route = (uint8_t *)malloc((size_t)T * B + 1);
    for (int i = 0; i < T * B; ++i) route[i] = (uint8_t)((i * 7 + 3) % 3 != 0);
    double *out = (double *)malloc(sizeof(double) * ((size_t)T * d_model + 1));
    double *h = (double *)malloc(sizeof(double) * ((size_t)T * d_inter + 1));
    double *g = (double *)malloc(sizeof(double) * ((size_t)T * d_inter + 1));
    int rc = 0;
    for (int mode = 0; mode < 2; ++mode) {
        rc |= oracle_mlpmoe_forward(x, Wg, Wu, Wd, off, alpha, mask, T, d_model, d_inter, B, mode, out);
        rc |= oracle_mlpmoe_forward_routed(x, Wg, Wu, Wd, off, alpha, mask, route, T, d_model, d_inter, B, mode, out);
        rc |= oracle_mlpmoe_hidden(x, Wg, Wu, off, alpha, mask, T, d_model, d_inter, B, mode, h, g, g, NULL, NULL);
    }
    rc |= oracle_dense_swiglu(x, Wg, Wu, Wd, T, d_model, d_inter, out);
    free(x); free(Wg); free(Wu); free(Wd); free(alpha); free(route); free(out); free(h); free(g);
    return rc;
}

int main(void)
{
    const int32_t off_a[] = {0, 33, 33, 77, 130};
    const uint8_t mask_a[] = {1, 1, 0, 1};
    const int32_t off_b[] = {0, 5};
    const uint8_t mask_b[] = {1};
    const int32_t off_c[] = {0, 0, 0};
    const uint8_t mask_c[] = {1, 0};
    int rc = 0;
    rc |= run_case(7, 50, off_a, mask_a, 4);
    rc |= run_case(1, 3, off_b, mask_b, 1);
    rc |= run_case(0, 8, off_a, mask_a, 4);       /* no tokens */
    rc |= run_case(5, 8, off_c, mask_c, 2);       /* no neurons */
    /* rejected arguments must be rejected before anything is touched */
    const int32_t bad[] = {0, 9, 4};
    double dummy[4];
    float f[4] = {0};
    if (oracle_mlpmoe_forward(f, f, f, f, bad, f, mask_c, 1, 1, 4, 2, 0, dummy) == 0) rc = 1;
    if (oracle_mlpmoe_forward(NULL, f, f, f, off_b, f, mask_b, 1, 1, 5, 1, 0, dummy) == 0) rc = 1;
    if (rc) {
        printf("FAILED rc=%d\n", rc);
        return 1;
    }
    printf("ok\n");
    return 0;
}
