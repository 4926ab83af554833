/*
 * CPU ORACLE for the neighbours of the inverse convolution inside one flow step
 * (Section 4.1: an Inv-Conv layer, an Actnorm layer and a 1 x 1 convolution; the
 * log-determinants of Section 4).  TEST INFRASTRUCTURE ONLY: plain definitions in
 * double that the GPU library is checked against.  Shares no code with the HIP
 * path; nothing in the product may call it.
 *
 *   Actnorm        a[n][c][r][q] = s[c] * x[n][c][r][q] + b[c]       (per-channel scale and bias)
 *   1 x 1 conv     z[n][o][r][q] = sum_i Q[o][i] * a[n][i][r][q]     (channel mixing, Q is C x C)
 *
 * Both act on every pixel independently, so their Jacobians are block diagonal:
 *   log|det da/dx| = H*W*sum_c log|s[c]|,   log|det dz/da| = H*W*log|det Q|   (one image).
 * Backward passes are the transposes of these linear maps; parameter gradients are
 * sums over batch and pixels.
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>

static inline size_t at(int C, int H, int W, int n, int ch, int r, int c)
{
    return (((size_t)n * C + ch) * H + r) * W + c;
}

void oracle_actnorm_fwd(const double *x, const double *s, const double *b, double *a,
                        int B, int C, int H, int W)
{
    for (int n = 0; n < B; ++n)
        for (int c = 0; c < C; ++c)
            for (int r = 0; r < H; ++r)
                for (int q = 0; q < W; ++q)
                    a[at(C, H, W, n, c, r, q)] = s[c] * x[at(C, H, W, n, c, r, q)] + b[c];
}

/* given ga = dL/da:  dL/dx = s * ga,  dL/ds[c] = sum ga * x,  dL/db[c] = sum ga */
void oracle_actnorm_bwd(const double *x, const double *s, const double *ga,
                        double *gx, double *gs, double *gb, int B, int C, int H, int W)
{
    for (int c = 0; c < C; ++c) {
        double acc_s = 0.0, acc_b = 0.0;
        for (int n = 0; n < B; ++n)
            for (int r = 0; r < H; ++r)
                for (int q = 0; q < W; ++q) {
                    const size_t p = at(C, H, W, n, c, r, q);
                    gx[p] = s[c] * ga[p];
                    acc_s += ga[p] * x[p];
                    acc_b += ga[p];
                }
        gs[c] = acc_s;
        gb[c] = acc_b;
    }
}

double oracle_actnorm_logdet(const double *s, int C, int H, int W)
{
    double acc = 0.0;
    for (int c = 0; c < C; ++c)
        acc += log(fabs(s[c]));
    return (double)H * (double)W * acc;
}

void oracle_conv1x1_fwd(const double *a, const double *Q, double *z, int B, int C, int H, int W)
{
    for (int n = 0; n < B; ++n)
        for (int o = 0; o < C; ++o)
            for (int r = 0; r < H; ++r)
                for (int q = 0; q < W; ++q) {
                    double acc = 0.0;
                    for (int i = 0; i < C; ++i)
                        acc += Q[(size_t)o * C + i] * a[at(C, H, W, n, i, r, q)];
                    z[at(C, H, W, n, o, r, q)] = acc;
                }
}

/* given gz = dL/dz:  dL/da[i] = sum_o Q[o][i] gz[o]  per pixel,  dL/dQ[o][i] = sum over batch and pixels of gz[o] * a[i] */
void oracle_conv1x1_bwd(const double *a, const double *Q, const double *gz,
                        double *ga, double *gQ, int B, int C, int H, int W)
{
    for (int n = 0; n < B; ++n)
        for (int i = 0; i < C; ++i)
            for (int r = 0; r < H; ++r)
                for (int q = 0; q < W; ++q) {
                    double acc = 0.0;
                    for (int o = 0; o < C; ++o)
                        acc += Q[(size_t)o * C + i] * gz[at(C, H, W, n, o, r, q)];
                    ga[at(C, H, W, n, i, r, q)] = acc;
                }
    for (int o = 0; o < C; ++o)
        for (int i = 0; i < C; ++i) {
            double acc = 0.0;
            for (int n = 0; n < B; ++n)
                for (int r = 0; r < H; ++r)
                    for (int q = 0; q < W; ++q)
                        acc += gz[at(C, H, W, n, o, r, q)] * a[at(C, H, W, n, i, r, q)];
            gQ[(size_t)o * C + i] = acc;
        }
}

/* H*W*log|det Q| by Gaussian elimination with partial pivoting; -inf for a singular Q */
double oracle_conv1x1_logdet(const double *Q, int C, int H, int W)
{
    double *m = (double *)malloc(sizeof(double) * (size_t)C * C);
    if (!m)
        return NAN;
    for (int e = 0; e < C * C; ++e)
        m[e] = Q[e];
    double acc = 0.0;
    for (int col = 0; col < C; ++col) {
        int piv = col;
        for (int r = col + 1; r < C; ++r)
            if (fabs(m[r * C + col]) > fabs(m[piv * C + col]))
                piv = r;
        if (m[piv * C + col] == 0.0) {
            free(m);
            return -INFINITY;
        }
        if (piv != col)
            for (int c = 0; c < C; ++c) {
                const double t = m[col * C + c];
                m[col * C + c] = m[piv * C + c];
                m[piv * C + c] = t;
            }
        acc += log(fabs(m[col * C + col]));
        for (int r = col + 1; r < C; ++r) {
            const double f = m[r * C + col] / m[col * C + col];
            for (int c = col; c < C; ++c)
                m[r * C + c] -= f * m[col * C + c];
        }
    }
    free(m);
    return (double)H * (double)W * acc;
}
