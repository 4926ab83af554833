// Determinant and inverse of an N x N matrix, N <= 4, by cofactors (no pivoting, no branches): what a wave
// needs of the 1 x 1 convolution's matrix Q when a flow step (Section 4.1) of few channels prepares its own
// channel maps instead of reading them from a set-up launch.  Double arithmetic; a singular matrix gives
// inf / NaN in the inverse, as the set-up launch does.
#pragma once

namespace invconv {

template <int N>
__host__ __device__ inline double small_det_inv(const double (&a)[N][N], double (&inv)[N][N])
{
    static_assert(N >= 1 && N <= 4, "cofactor formulas up to 4 x 4");
    if constexpr (N == 1) {
        inv[0][0] = 1.0 / a[0][0];
        return a[0][0];
    } else if constexpr (N == 2) {
        const double det = a[0][0] * a[1][1] - a[0][1] * a[1][0];
        const double r = 1.0 / det;
        inv[0][0] = a[1][1] * r;
        inv[0][1] = -a[0][1] * r;
        inv[1][0] = -a[1][0] * r;
        inv[1][1] = a[0][0] * r;
        return det;
    } else if constexpr (N == 3) {
        // adj[i][j] = cofactor of a[j][i]
        double adj[3][3];
#pragma unroll
        for (int i = 0; i < 3; ++i)
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                const int r0 = (j + 1) % 3, r1 = (j + 2) % 3, c0 = (i + 1) % 3, c1 = (i + 2) % 3;
                adj[i][j] = a[r0][c0] * a[r1][c1] - a[r0][c1] * a[r1][c0];     // cyclic indices carry the sign
            }
        const double det = a[0][0] * adj[0][0] + a[0][1] * adj[1][0] + a[0][2] * adj[2][0];
        const double r = 1.0 / det;
#pragma unroll
        for (int i = 0; i < 3; ++i)
#pragma unroll
            for (int j = 0; j < 3; ++j)
                inv[i][j] = adj[i][j] * r;
        return det;
    } else {
        // Laplace expansion along the first two rows: 2 x 2 minors of rows 0,1 (s) and of rows 2,3 (c)
        const double s0 = a[0][0] * a[1][1] - a[1][0] * a[0][1], s1 = a[0][0] * a[1][2] - a[1][0] * a[0][2];
        const double s2 = a[0][0] * a[1][3] - a[1][0] * a[0][3], s3 = a[0][1] * a[1][2] - a[1][1] * a[0][2];
        const double s4 = a[0][1] * a[1][3] - a[1][1] * a[0][3], s5 = a[0][2] * a[1][3] - a[1][2] * a[0][3];
        const double c5 = a[2][2] * a[3][3] - a[3][2] * a[2][3], c4 = a[2][1] * a[3][3] - a[3][1] * a[2][3];
        const double c3 = a[2][1] * a[3][2] - a[3][1] * a[2][2], c2 = a[2][0] * a[3][3] - a[3][0] * a[2][3];
        const double c1 = a[2][0] * a[3][2] - a[3][0] * a[2][2], c0 = a[2][0] * a[3][1] - a[3][0] * a[2][1];
        const double det = s0 * c5 - s1 * c4 + s2 * c3 + s3 * c2 - s4 * c1 + s5 * c0;
        const double r = 1.0 / det;
        inv[0][0] = (a[1][1] * c5 - a[1][2] * c4 + a[1][3] * c3) * r;
        inv[0][1] = (-a[0][1] * c5 + a[0][2] * c4 - a[0][3] * c3) * r;
        inv[0][2] = (a[3][1] * s5 - a[3][2] * s4 + a[3][3] * s3) * r;
        inv[0][3] = (-a[2][1] * s5 + a[2][2] * s4 - a[2][3] * s3) * r;
        inv[1][0] = (-a[1][0] * c5 + a[1][2] * c2 - a[1][3] * c1) * r;
        inv[1][1] = (a[0][0] * c5 - a[0][2] * c2 + a[0][3] * c1) * r;
        inv[1][2] = (-a[3][0] * s5 + a[3][2] * s2 - a[3][3] * s1) * r;
        inv[1][3] = (a[2][0] * s5 - a[2][2] * s2 + a[2][3] * s1) * r;
        inv[2][0] = (a[1][0] * c4 - a[1][1] * c2 + a[1][3] * c0) * r;
        inv[2][1] = (-a[0][0] * c4 + a[0][1] * c2 - a[0][3] * c0) * r;
        inv[2][2] = (a[3][0] * s4 - a[3][1] * s2 + a[3][3] * s0) * r;
        inv[2][3] = (-a[2][0] * s4 + a[2][1] * s2 - a[2][3] * s0) * r;
        inv[3][0] = (-a[1][0] * c3 + a[1][1] * c1 - a[1][2] * c0) * r;
        inv[3][1] = (a[0][0] * c3 - a[0][1] * c1 + a[0][2] * c0) * r;
        inv[3][2] = (-a[3][0] * s3 + a[3][1] * s1 - a[3][2] * s0) * r;
        inv[3][3] = (a[2][0] * s3 - a[2][1] * s1 + a[2][2] * s0) * r;
        return det;
    }
}

}  // namespace invconv
