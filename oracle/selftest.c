/*
 * Sanitizer self-test of the CPU oracle (TEST INFRASTRUCTURE ONLY).  Built by tests/test_oracle_sanitizers.py
 * with -fsanitize=address,undefined together with the two oracle sources and run as a plain executable: every
 * oracle routine is called on small odd-sized inputs (k larger than the image, one row, one column, several
 * channels), so that an out-of-bounds index or undefined arithmetic in the oracle aborts the run.  The only
 * values checked here are round trips; the pins proper live in the Python tests.
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

void oracle_conv(const double *, const double *, double *, int, int, int, int, int, int);
void oracle_invconv_fwd(const double *, const double *, double *, int, int, int, int, int, int);
void oracle_invconv_bwd_dy(const double *, const double *, double *, int, int, int, int, int, int);
void oracle_invconv_bwd_dw(const double *, const double *, double *, int, int, int, int, int, int);
void oracle_conv_bwd_dx(const double *, const double *, double *, int, int, int, int, int, int);
void oracle_conv_bwd_dw(const double *, const double *, double *, int, int, int, int, int, int);
double oracle_invconv_logdet(const double *, int, int, int, int);
void oracle_actnorm_fwd(const double *, const double *, const double *, double *, int, int, int, int);
void oracle_actnorm_bwd(const double *, const double *, const double *, double *, double *, double *, int, int, int, int);
double oracle_actnorm_logdet(const double *, int, int, int);
void oracle_conv1x1_fwd(const double *, const double *, double *, int, int, int, int);
void oracle_conv1x1_bwd(const double *, const double *, const double *, double *, double *, int, int, int, int);
double oracle_conv1x1_logdet(const double *, int, int, int);

static unsigned long long state = 88172645463325252ull;
static double rnd(void)
{
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return (double)(state >> 11) / 9007199254740992.0 - 0.5;
}

static int one_shape(int B, int C, int H, int W, int k)
{
    const size_t n = (size_t)B * C * H * W, p = (size_t)C * C * k * k;
    double *y = malloc(n * sizeof(double)), *x = malloc(n * sizeof(double)), *y2 = malloc(n * sizeof(double));
    double *g = malloc(n * sizeof(double)), *v = malloc(n * sizeof(double)), *a = malloc(n * sizeof(double));
    double *w = malloc(p * sizeof(double)), *dw = malloc(p * sizeof(double));
    double *s = malloc(C * sizeof(double)), *b = malloc(C * sizeof(double)), *Q = malloc((size_t)C * C * sizeof(double));
    double *gs = malloc(C * sizeof(double)), *gb = malloc(C * sizeof(double)), *gQ = malloc((size_t)C * C * sizeof(double));
    if (!y || !x || !y2 || !g || !v || !a || !w || !dw || !s || !b || !Q || !gs || !gb || !gQ)
        return 2;
    for (size_t i = 0; i < n; ++i) {
        y[i] = rnd();
        g[i] = rnd();
    }
    for (size_t i = 0; i < p; ++i)
        w[i] = 0.2 * rnd();
    for (int c = 0; c < C; ++c) {
        w[(((size_t)c * C + c) * k + (k - 1)) * k + (k - 1)] = 1.0 + 0.5 * rnd();
        s[c] = 1.0 + rnd();
        b[c] = rnd();
        for (int d = 0; d < C; ++d)
            Q[c * C + d] = (c == d ? 1.0 : 0.0) + 0.2 * rnd();
    }
    int bad = 0;
    oracle_invconv_fwd(y, w, x, B, C, H, W, k, 1);
    oracle_conv(x, w, y2, B, C, H, W, k, 1);
    for (size_t i = 0; i < n; ++i)
        bad |= fabs(y2[i] - y[i]) > 1e-9;
    oracle_invconv_bwd_dy(g, w, v, B, C, H, W, k, 2);
    oracle_invconv_bwd_dw(x, v, dw, B, C, H, W, k, 2);
    oracle_conv_bwd_dx(g, w, v, B, C, H, W, k, 1);
    oracle_conv_bwd_dw(x, g, dw, B, C, H, W, k, 1);
    bad |= !isfinite(oracle_invconv_logdet(w, C, H, W, k));
    oracle_actnorm_fwd(x, s, b, a, B, C, H, W);
    oracle_conv1x1_fwd(a, Q, y2, B, C, H, W);
    oracle_conv1x1_bwd(a, Q, g, v, gQ, B, C, H, W);
    oracle_actnorm_bwd(x, s, v, y2, gs, gb, B, C, H, W);
    bad |= !isfinite(oracle_actnorm_logdet(s, C, H, W)) || !isfinite(oracle_conv1x1_logdet(Q, C, H, W));
    free(y); free(x); free(y2); free(g); free(v); free(a); free(w); free(dw);
    free(s); free(b); free(Q); free(gs); free(gb); free(gQ);
    return bad;
}

int main(void)
{
    static const int shapes[][5] = {{1, 1, 1, 1, 1}, {2, 3, 4, 5, 3}, {1, 2, 2, 2, 5}, {1, 4, 1, 7, 3},
                                    {1, 4, 7, 1, 3}, {3, 5, 6, 3, 2}, {1, 12, 5, 5, 3}};
    for (unsigned i = 0; i < sizeof(shapes) / sizeof(shapes[0]); ++i) {
        const int r = one_shape(shapes[i][0], shapes[i][1], shapes[i][2], shapes[i][3], shapes[i][4]);
        if (r) {
            printf("selftest: shape %u failed (%d)\n", i, r);
            return 1;
        }
    }
    printf("selftest: ok\n");
    return 0;
}
