/*
 * CPU ORACLE for the inverse of a causally masked k x k convolution and its
 * backpropagation.  TEST INFRASTRUCTURE ONLY: this file is the slow, plain
 * definition the GPU library is checked against.  It shares no code with the
 * HIP path and nothing in the product may call it.
 *
 * All arithmetic is in double.  Activations are [B][C][H][W], kernels are
 * [C_out][C_in][k][k] (Algorithm 1's K[c, k_c, ., .]).  Tap (a,b) multiplies
 * the input pixel (r-(k-1)+a, c-(k-1)+b): the image is padded with k-1 zeros on
 * the top and left and the bottom-right tap (k-1,k-1) sits on the current pixel
 * (Section 3, Eq. 1, supplement "Input Padding and Kernel Masking").
 *
 * The paper treats one channel with a unit bottom-right tap.  For C channels
 * the bottom-right tap becomes a C x C block that is lower triangular in
 * (out, in) with a non-zero diagonal; entries above that diagonal are treated
 * as zero whatever the array holds ("masked").  With pixels ordered row-major
 * and channels innermost, the convolution matrix M is then lower triangular
 * with the block diagonals on its diagonal (Section 3, second paragraph).
 *
 * Pixels are visited in row-major order, a topological order of the paper's
 * partial order p <= q that differs from the anti-diagonal order a parallel
 * implementation uses.
 */
#include <math.h>
#include <stddef.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* effective kernel entry: masked entries read as zero */
static inline double eff(const double *w, int C, int k, int o, int i, int a, int b)
{
    if (a == k - 1 && b == k - 1 && i > o)
        return 0.0;
    return w[(((size_t)o * C + i) * k + a) * k + b];
}

static inline size_t at(int C, int H, int W, int n, int ch, int r, int c)
{
    return (((size_t)n * C + ch) * H + r) * W + c;
}

/* Eq. 1 with channels: y = conv_w(x), zero padding top/left. */
void oracle_conv(const double *x, const double *w, double *y,
                 int B, int C, int H, int W, int k, int threads)
{
    (void)threads;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int n = 0; n < B; ++n)
        for (int o = 0; o < C; ++o)
            for (int r = 0; r < H; ++r)
                for (int c = 0; c < W; ++c) {
                    double acc = 0.0;
                    for (int i = 0; i < C; ++i)
                        for (int a = 0; a < k; ++a)
                            for (int b = 0; b < k; ++b) {
                                int rr = r - (k - 1) + a, cc = c - (k - 1) + b;
                                if (rr < 0 || cc < 0)
                                    continue;
                                acc += eff(w, C, k, o, i, a, b) * x[at(C, H, W, n, i, rr, cc)];
                            }
                    y[at(C, H, W, n, o, r, c)] = acc;
                }
}

/*
 * Gradients of the convolution itself (the sampling direction only needs plain
 * convolutions, Section 4.3).  y = M x is linear in x and in w, so with g = dL/dy
 *   dL/dx = M^T g:  dL/dx[n][i][r][c] = sum_{o,a,b} w[o][i][a][b] g[n][o][r+(k-1)-a][c+(k-1)-b]
 * over the output pixels inside the image that read input pixel (r, c) through tap
 * (a, b), and
 *   dL/dw[o][i][a][b] = sum_{n,r,c} g[n][o][r][c] x[n][i][r-(k-1)+a][c-(k-1)+b],
 * masked entries 0.
 */
void oracle_conv_bwd_dx(const double *g, const double *w, double *dx,
                        int B, int C, int H, int W, int k, int threads)
{
    (void)threads;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int n = 0; n < B; ++n)
        for (int i = 0; i < C; ++i)
            for (int r = 0; r < H; ++r)
                for (int c = 0; c < W; ++c) {
                    double acc = 0.0;
                    for (int o = 0; o < C; ++o)
                        for (int a = 0; a < k; ++a)
                            for (int b = 0; b < k; ++b) {
                                int rr = r + (k - 1) - a, cc = c + (k - 1) - b;
                                if (rr >= H || cc >= W)
                                    continue;
                                acc += eff(w, C, k, o, i, a, b) * g[at(C, H, W, n, o, rr, cc)];
                            }
                    dx[at(C, H, W, n, i, r, c)] = acc;
                }
}

void oracle_conv_bwd_dw(const double *x, const double *g, double *dw,
                        int B, int C, int H, int W, int k, int threads)
{
    (void)threads;
    int P = C * C * k * k;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int e = 0; e < P; ++e) {
        int b = e % k, a = (e / k) % k, i = (e / (k * k)) % C, o = e / (k * k * C);
        double acc = 0.0;
        if (!(a == k - 1 && b == k - 1 && i > o)) {
            for (int n = 0; n < B; ++n)
                for (int r = 0; r < H; ++r)
                    for (int c = 0; c < W; ++c) {
                        int rr = r - (k - 1) + a, cc = c - (k - 1) + b;
                        if (rr < 0 || cc < 0)
                            continue;
                        acc += g[at(C, H, W, n, o, r, c)] * x[at(C, H, W, n, i, rr, cc)];
                    }
        }
        dw[e] = acc;
    }
}

/*
 * Inverse convolution: solve conv_w(x) = y for x by forward substitution,
 *   x_q = ( y_q - sum_{r in Delta(q)} W_{(k,k)-q+r} x_r ) / W_{k,k}
 * (the rearranged Eq. 1 used in the proofs of Theorems 1 and 2), extended to
 * channels: inside a pixel the channels are solved in increasing order.
 */
void oracle_invconv_fwd(const double *y, const double *w, double *x,
                        int B, int C, int H, int W, int k, int threads)
{
    (void)threads;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int n = 0; n < B; ++n)
        for (int r = 0; r < H; ++r)
            for (int c = 0; c < W; ++c)
                for (int o = 0; o < C; ++o) {
                    double acc = y[at(C, H, W, n, o, r, c)];
                    for (int i = 0; i < C; ++i)
                        for (int a = 0; a < k; ++a)
                            for (int b = 0; b < k; ++b) {
                                if (a == k - 1 && b == k - 1)
                                    continue;
                                int rr = r - (k - 1) + a, cc = c - (k - 1) + b;
                                if (rr < 0 || cc < 0)
                                    continue;
                                acc -= eff(w, C, k, o, i, a, b) * x[at(C, H, W, n, i, rr, cc)];
                            }
                    for (int i = 0; i < o; ++i)
                        acc -= eff(w, C, k, o, i, k - 1, k - 1) * x[at(C, H, W, n, i, r, c)];
                    x[at(C, H, W, n, o, r, c)] = acc / eff(w, C, k, o, o, k - 1, k - 1);
                }
}

/*
 * Input gradient (Eq. 2 with Theorem 1): dL/dy_p = sum_q dL/dx_q dx_q/dy_p.
 * dx_q/dy_p are the entries of M^{-1}, so dL/dy = M^{-T} g, obtained by
 * back-substitution on the transposed system in reverse row-major order:
 *   v_p = ( g_p - sum_{q : p in Delta(q)} W_{(k,k)-q+p} v_q ) / W_{k,k}.
 */
void oracle_invconv_bwd_dy(const double *g, const double *w, double *v,
                           int B, int C, int H, int W, int k, int threads)
{
    (void)threads;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int n = 0; n < B; ++n)
        for (int r = H - 1; r >= 0; --r)
            for (int c = W - 1; c >= 0; --c)
                for (int i = C - 1; i >= 0; --i) {
                    double acc = g[at(C, H, W, n, i, r, c)];
                    for (int o = 0; o < C; ++o)
                        for (int a = 0; a < k; ++a)
                            for (int b = 0; b < k; ++b) {
                                if (a == k - 1 && b == k - 1)
                                    continue;
                                /* output pixel q that reads p=(r,c) through tap (a,b) */
                                int qr = r + (k - 1) - a, qc = c + (k - 1) - b;
                                if (qr >= H || qc >= W)
                                    continue;
                                acc -= eff(w, C, k, o, i, a, b) * v[at(C, H, W, n, o, qr, qc)];
                            }
                    for (int o = i + 1; o < C; ++o)
                        acc -= eff(w, C, k, o, i, k - 1, k - 1) * v[at(C, H, W, n, o, r, c)];
                    v[at(C, H, W, n, i, r, c)] = acc / eff(w, C, k, i, i, k - 1, k - 1);
                }
}

/*
 * Weight gradient (Eq. 4 with Theorem 2).  Contracting Theorem 2's recursion
 * for dx_q/dW_a with dL/dx gives
 *   dL/dW[o][i][a][b] = - sum_{n,r,c} v[n][o][r][c] * x[n][i][r-(k-1)+a][c-(k-1)+b]
 * with v = dL/dy, summed over batch and pixels; masked entries are 0.
 */
void oracle_invconv_bwd_dw(const double *x, const double *v, double *dw,
                           int B, int C, int H, int W, int k, int threads)
{
    (void)threads;
    int P = C * C * k * k;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int e = 0; e < P; ++e) {
        int b = e % k, a = (e / k) % k, i = (e / (k * k)) % C, o = e / (k * k * C);
        double acc = 0.0;
        if (!(a == k - 1 && b == k - 1 && i > o)) {
            for (int n = 0; n < B; ++n)
                for (int r = 0; r < H; ++r)
                    for (int c = 0; c < W; ++c) {
                        int rr = r - (k - 1) + a, cc = c - (k - 1) + b;
                        if (rr < 0 || cc < 0)
                            continue;
                        acc += v[at(C, H, W, n, o, r, c)] * x[at(C, H, W, n, i, rr, cc)];
                    }
            acc = -acc;
        }
        dw[e] = acc;
    }
}

/*
 * log |det d x / d y| of the inverse convolution for one image (Section 4):
 * M is triangular, so det M = prod over pixels and channels of the diagonal of
 * the bottom-right tap, and the inverse map has the negative log-determinant.
 * Exactly 0 when that diagonal is 1.
 */
double oracle_invconv_logdet(const double *w, int C, int H, int W, int k)
{
    double s = 0.0;
    for (int c = 0; c < C; ++c)
        s += log(fabs(eff(w, C, k, c, c, k - 1, k - 1)));
    return -(double)H * (double)W * s;
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
