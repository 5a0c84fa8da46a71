/*
 * CPU oracle for the branched SwiGLU MLP forward of MLPMoE.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, double-precision
 * evaluation of the definition and exists only so that tests, the smoke check
 * and the benchmark's CPU-baseline leg can compare the GPU library against it.
 * The GPU library never calls it and shares no code with it.
 *
 * What it computes (Sec. 3.1):
 *     branch_b(x) = alpha_b * W_down^(b) [ phi(W_gate^(b) x) (.) W_up^(b) x ]
 *     MLPMoE(x)   = sum_b branch_b(x)
 * with phi = SiLU, phi(z) = z / (1 + exp(-z)); the branches are contiguous
 * slices [off[b], off[b+1]) of the intermediate dimension.  A branch whose
 * active flag is 0 is skipped altogether (Sec. 3.3: pruned branches), so
 * non-finite weights inside it cannot reach the output.
 *
 * Layouts (row-major): x [T,d_model]; W_gate, W_up [d_inter,d_model] (one row
 * per neuron); W_down [d_model,d_inter] (one column per neuron);
 * out [T,d_model] double.  Inputs are the stored values widened exactly to
 * float (bf16 -> float is exact), all sums are taken in double.
 *
 * mode 0 ("exact"):    no intermediate rounding at all.
 * mode 1 ("contract"): the bf16 pipeline's single rounding point is reproduced:
 *     the gated intermediate of neuron j in branch b, scaled by alpha_b, is
 *     formed in float and rounded once to bf16 (nearest-even) before the down
 *     projection; alpha_b is therefore not applied a second time.  Everything
 *     else stays in double.  This is the precision the GPU kernels take that
 *     rounding decision in.
 *
 * Pins (tests/test_oracle_pins.py): dense-MLP identity of Sec. 2.2 / 3.1 via a
 * library fp64 matmul, per-branch brute force, linearity in alpha, mask == alpha
 * 0 == row deletion, neuron removal == zeroed rows, permutation invariance,
 * one-hot inputs, SiLU special values.  The paper prints no forward values, so
 * there is no printed-number pin for this function.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double silu_d(double z) { return z / (1.0 + exp(-z)); }

/* float -> bf16 -> float, round to nearest even; NaN stays NaN. */
static float round_to_bf16(float v)
{
    uint32_t u;
    memcpy(&u, &v, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) {
        u |= 0x00400000u;
        u &= 0xffff0000u;
    } else {
        u += 0x7fffu + ((u >> 16) & 1u);
        u &= 0xffff0000u;
    }
    memcpy(&v, &u, 4);
    return v;
}

/* One token: out_row[0..d_model) = MLPMoE(x_row).  h is scratch of d_inter doubles. */
static void forward_token(const float *x_row, const float *Wg, const float *Wu, const float *Wd,
                          const int32_t *off, const float *alpha, const uint8_t *active,
                          int d_model, int d_inter, int B, int mode, double *h, double *out_row)
{
    for (int m = 0; m < d_model; ++m) out_row[m] = 0.0;
    for (int b = 0; b < B; ++b) {
        if (!active[b]) continue;
        const int j0 = off[b], j1 = off[b + 1];
        /* gated intermediate of this branch: h_j = SiLU(<Wg_j,x>) * <Wu_j,x> */
        for (int j = j0; j < j1; ++j) {
            const float *g_row = Wg + (size_t)j * d_model;
            const float *u_row = Wu + (size_t)j * d_model;
            double g = 0.0, u = 0.0;
            for (int k = 0; k < d_model; ++k) {
                g += (double)x_row[k] * (double)g_row[k];
                u += (double)x_row[k] * (double)u_row[k];
            }
            if (mode == 0) {
                h[j] = silu_d(g) * u;
            } else {
                /* rounding decision taken in float, as the bf16 pipeline does */
                float gf = (float)g, uf = (float)u;
                float s = gf / (1.0f + expf(-gf));
                float hv = alpha[b] * (s * uf);
                h[j] = (double)round_to_bf16(hv);
            }
        }
        /* down projection of the branch, then alpha_b and the sum over branches */
        for (int m = 0; m < d_model; ++m) {
            const float *d_row = Wd + (size_t)m * d_inter;
            double acc = 0.0;
            for (int j = j0; j < j1; ++j) acc += h[j] * (double)d_row[j];
            out_row[m] += (mode == 0) ? (double)alpha[b] * acc : acc;
        }
    }
}

/*
 * Returns 0 on success, -1 on a bad argument, -2 if scratch cannot be allocated.
 * Tokens are independent; with OpenMP they are spread over the host's threads.
 */
int oracle_mlpmoe_forward(const float *x, const float *Wg, const float *Wu, const float *Wd,
                          const int32_t *off, const float *alpha, const uint8_t *active,
                          int T, int d_model, int d_inter, int B, int mode, double *out)
{
    if (!x || !Wg || !Wu || !Wd || !off || !alpha || !active || !out) return -1;
    if (T < 0 || d_model <= 0 || d_inter < 0 || B <= 0) return -1;
    if (off[0] != 0 || off[B] != d_inter) return -1;
    for (int b = 0; b < B; ++b)
        if (off[b + 1] < off[b]) return -1;
    int fail = 0;
#pragma omp parallel
    {
        double *h = (double *)malloc(sizeof(double) * (size_t)(d_inter > 0 ? d_inter : 1));
        if (!h) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 1)
            for (int t = 0; t < T; ++t)
                forward_token(x + (size_t)t * d_model, Wg, Wu, Wd, off, alpha, active, d_model,
                              d_inter, B, mode, h, out + (size_t)t * d_model);
        }
        free(h);
    }
    return fail ? -2 : 0;
}

/*
 * Per-token routing over branches (the paper names dynamic routing as the natural extension of the
 * branch structure, Sec. 7 / Sec. 8, without defining it; reading taken here): every token t has
 * its own set of branches, route[t*B + b] != 0, and
 *     out_t = sum over { b : active[b] and route[t][b] } of alpha_b W_down^(b)[SiLU(W_gate^(b) x_t) (.) W_up^(b) x_t].
 * That is the forward above with the branch mask replaced, token by token, by active AND route_t.
 */
int oracle_mlpmoe_forward_routed(const float *x, const float *Wg, const float *Wu, const float *Wd,
                                 const int32_t *off, const float *alpha, const uint8_t *active,
                                 const uint8_t *route, int T, int d_model, int d_inter, int B, int mode,
                                 double *out)
{
    if (!x || !Wg || !Wu || !Wd || !off || !alpha || !active || !route || !out) return -1;
    if (T < 0 || d_model <= 0 || d_inter < 0 || B <= 0 || B > 4096) return -1;
    if (off[0] != 0 || off[B] != d_inter) return -1;
    for (int b = 0; b < B; ++b)
        if (off[b + 1] < off[b]) return -1;
    int fail = 0;
#pragma omp parallel
    {
        double *h = (double *)malloc(sizeof(double) * (size_t)(d_inter > 0 ? d_inter : 1));
        uint8_t *eff = (uint8_t *)malloc((size_t)B);
        if (!h || !eff) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 1)
            for (int t = 0; t < T; ++t) {
                for (int b = 0; b < B; ++b) eff[b] = (uint8_t)(active[b] && route[(size_t)t * B + b]);
                forward_token(x + (size_t)t * d_model, Wg, Wu, Wd, off, alpha, eff, d_model, d_inter, B,
                              mode, h, out + (size_t)t * d_model);
            }
        }
        free(h);
        free(eff);
    }
    return fail ? -2 : 0;
}

/*
 * The gated intermediate on its own (the bracket of Sec. 3.1 times alpha_b), for tests that look at
 * the bf16 pipeline's single rounding point directly instead of through the down projection:
 *     h[t][j] = alpha_b * SiLU(g) * u,   g = <W_gate[j], x_t>,  u = <W_up[j], x_t>,  b = branch of j
 * mode 0: that product in double.  mode 1: formed in float and rounded once to bf16, exactly as the
 * contract mode of oracle_mlpmoe_forward does (so that forward(contract) = h(contract) W_down^T).
 * Neurons of inactive branches get 0.  Optional outputs (NULL to skip), each [T, d_inter]:
 *     g, u          the two dot products in double
 *     abs_g, abs_u  sum_k |x_k| |w_k| of the same dot products: the scale of the rounding error of
 *                   any floating-point evaluation of them, which decides how close to a bf16
 *                   rounding boundary a value must lie before two correct evaluations may round it
 *                   to different neighbours.
 */
int oracle_mlpmoe_hidden(const float *x, const float *Wg, const float *Wu, const int32_t *off,
                         const float *alpha, const uint8_t *active, int T, int d_model, int d_inter, int B,
                         int mode, double *h, double *g_out, double *u_out, double *abs_g, double *abs_u)
{
    if (!x || !Wg || !Wu || !off || !alpha || !active || !h) return -1;
    if (T < 0 || d_model <= 0 || d_inter < 0 || B <= 0) return -1;
    if (off[0] != 0 || off[B] != d_inter) return -1;
    for (int b = 0; b < B; ++b)
        if (off[b + 1] < off[b]) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int t = 0; t < T; ++t) {
        const float *x_row = x + (size_t)t * d_model;
        for (int b = 0; b < B; ++b) {
            for (int j = off[b]; j < off[b + 1]; ++j) {
                const size_t o = (size_t)t * d_inter + j;
                const float *g_row = Wg + (size_t)j * d_model;
                const float *u_row = Wu + (size_t)j * d_model;
                double g = 0.0, u = 0.0, ag = 0.0, au = 0.0;
                if (active[b]) {
                    for (int k = 0; k < d_model; ++k) {
                        const double pg = (double)x_row[k] * (double)g_row[k];
                        const double pu = (double)x_row[k] * (double)u_row[k];
                        g += pg;
                        u += pu;
                        ag += fabs(pg);
                        au += fabs(pu);
                    }
                }
                double hv = 0.0;
                if (active[b]) {
                    if (mode == 0) {
                        hv = (double)alpha[b] * (silu_d(g) * u);
                    } else {
                        float gf = (float)g, uf = (float)u;
                        float s = gf / (1.0f + expf(-gf));
                        hv = (double)round_to_bf16(alpha[b] * (s * uf));
                    }
                }
                h[o] = hv;
                if (g_out) g_out[o] = g;
                if (u_out) u_out[o] = u;
                if (abs_g) abs_g[o] = ag;
                if (abs_u) abs_u[o] = au;
            }
        }
    }
    return 0;
}

/* Dense SwiGLU MLP with no branch structure: W_down [ SiLU(W_gate x) (.) W_up x ]  (Sec. 2.2 identity,
 * right-hand side before slicing).  Kept separate from the branched code path on purpose. */
int oracle_dense_swiglu(const float *x, const float *Wg, const float *Wu, const float *Wd,
                        int T, int d_model, int d_inter, double *out)
{
    if (!x || !Wg || !Wu || !Wd || !out || T < 0 || d_model <= 0 || d_inter < 0) return -1;
    double *h = (double *)malloc(sizeof(double) * (size_t)(d_inter > 0 ? d_inter : 1));
    if (!h) return -2;
    for (int t = 0; t < T; ++t) {
        const float *xr = x + (size_t)t * d_model;
        for (int j = 0; j < d_inter; ++j) {
            double g = 0.0, u = 0.0;
            for (int k = 0; k < d_model; ++k) {
                g += (double)Wg[(size_t)j * d_model + k] * (double)xr[k];
                u += (double)Wu[(size_t)j * d_model + k] * (double)xr[k];
            }
            h[j] = silu_d(g) * u;
        }
        for (int m = 0; m < d_model; ++m) {
            double acc = 0.0;
            for (int j = 0; j < d_inter; ++j) acc += (double)Wd[(size_t)m * d_inter + j] * h[j];
            out[(size_t)t * d_model + m] = acc;
        }
    }
    free(h);
    return 0;
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}
