// Inverse of the lower-triangular current-pixel block of a many-channel kernel (17 .. 48 channels) by a whole
// workgroup, in 16 x 16 blocks.  gfx950 only.
//
// The folded form of the solve (Eq. 1 rearranged: x_p = Linv y_p - sum_tap Linv W_tap x_{p - tap}) needs Linv once
// per call.  Forward substitution with one thread per column is a chain of C dependent rows (48 channels: 8 us of
// one wave while the others wait).  In blocks, with X = L^-1:
//     X[c][c] = L[c][c]^-1                                   (three independent chains of 16 rows)
//     X[r][c] = -X[r][r] sum_{m = c}^{r-1} L[r][m] X[m][c]   (r > c: 16 x 16 x 16 products, one thread per entry)
// which for at most three blocks is five short stages between workgroup barriers.
#pragma once
#include <hip/hip_runtime.h>

namespace invconv {

constexpr int tri_inverse_tmp_floats() { return 3 * 256; }

// sL: [C][C] row-major, entries above the diagonal zero.  sX: the result, row stride ldx, rows and columns < C
// (entries above the diagonal are written as zeros).  sTmp: tri_inverse_tmp_floats() floats.  Every thread of the
// workgroup calls it (at least ceil(C / 16) waves); C a multiple of 4, 17 <= C <= 48.  Ends with a barrier.
template <int C>
__device__ __forceinline__ void tri_inverse_blocks(const float *sL, float *sX, int ldx, float *sTmp)
{
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    static_assert(C % 4 == 0 && C > 16 && C <= 48, "two or three blocks of 16");
    constexpr int NBK = (C + 15) / 16;
    const int tid = threadIdx.x, nt = blockDim.x, wave = tid >> 6, lane = tid & 63;
    // L and X as if padded with an identity to whole blocks
    auto Lat = [&](int o, int i) -> float { return (o < C && i < C) ? sL[o * C + i] : (o == i ? 1.0f : 0.0f); };
    auto Xat = [&](int o, int i) -> float { return (o < C && i < C) ? sX[o * ldx + i] : (o == i ? 1.0f : 0.0f); };

    // stage 1: the diagonal blocks, wave b, column j of the block by lane j with the column in registers
    if (wave < NBK && lane < 16) {
        const int b0 = 16 * wave, j = lane;
        float col[16];
#pragma unroll
        for (int o = 0; o < 16; ++o) {
            float part[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            float diag = 1.0f;
            if (b0 + o < C) {
#pragma unroll
                for (int m4 = 0; m4 <= o / 4; ++m4) {
                    const f32x4 row = *reinterpret_cast<const f32x4 *>(sL + (b0 + o) * C + b0 + 4 * m4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (4 * m4 + e < o)
                            part[e] += row[e] * col[4 * m4 + e];
                        else if (4 * m4 + e == o)
                            diag = row[e];
                    }
                }
            }
            const float sum = (part[0] + part[1]) + (part[2] + part[3]);
            const float rd = 1.0f / diag;
            col[o] = o < j ? 0.0f : (o == j ? rd : -sum * rd);
        }
        if (b0 + j < C) {
#pragma unroll
            for (int o = 0; o < 16; ++o)
                if (b0 + o < C)
                    sX[(b0 + o) * ldx + b0 + j] = col[o];
        }
    }
    // the blocks above the diagonal are zeros
    for (int idx = tid; idx < C * C; idx += nt) {
        const int o = idx / C, i = idx % C;
        if (i / 16 > o / 16)
            sX[o * ldx + i] = 0.0f;
    }
    __syncthreads();
    // stage 2: L[r][c] X[c][c] for (r, c) = (1, 0), (2, 1), (2, 0) into tmp 0, 1, 2
    constexpr int NP = NBK == 3 ? 3 : 1;
    for (int idx = tid; idx < NP * 256; idx += nt) {
        const int p = idx >> 8, i = (idx >> 4) & 15, jj = idx & 15;
        const int r = p == 0 ? 1 : 2, c = p == 1 ? 1 : 0;
        float s = 0.0f;
#pragma unroll
        for (int m = 0; m < 16; ++m)
            s += Lat(16 * r + i, 16 * c + m) * Xat(16 * c + m, 16 * c + jj);
        sTmp[idx] = s;
    }
    __syncthreads();
    // stage 3: X[1][0] = -X[1][1] tmp0, X[2][1] = -X[2][2] tmp1
    constexpr int NQ = NBK == 3 ? 2 : 1;
    for (int idx = tid; idx < NQ * 256; idx += nt) {
        const int p = idx >> 8, i = (idx >> 4) & 15, jj = idx & 15;
        const int r = p + 1, c = p;
        float s = 0.0f;
#pragma unroll
        for (int m = 0; m < 16; ++m)
            s += Xat(16 * r + i, 16 * r + m) * sTmp[p * 256 + m * 16 + jj];
        if (16 * r + i < C && 16 * c + jj < C)
            sX[(16 * r + i) * ldx + 16 * c + jj] = -s;
    }
    __syncthreads();
    if constexpr (NBK == 3) {
        // stage 4: tmp2 += L[2][1] X[1][0]
        for (int idx = tid; idx < 256; idx += nt) {
            const int i = (idx >> 4) & 15, jj = idx & 15;
            float s = sTmp[512 + idx];
#pragma unroll
            for (int m = 0; m < 16; ++m)
                s += Lat(32 + i, 16 + m) * Xat(16 + m, jj);
            sTmp[512 + idx] = s;
        }
        __syncthreads();
        // stage 5: X[2][0] = -X[2][2] tmp2
        for (int idx = tid; idx < 256; idx += nt) {
            const int i = (idx >> 4) & 15, jj = idx & 15;
            float s = 0.0f;
#pragma unroll
            for (int m = 0; m < 16; ++m)
                s += Xat(32 + i, 32 + m) * sTmp[512 + m * 16 + jj];
            if (32 + i < C)
                sX[(32 + i) * ldx + jj] = -s;
        }
        __syncthreads();
    }
}

}  // namespace invconv
