// Inverse and log|det| of a small matrix by one wave (gfx950): what the flow-step kernels need of the 1 x 1
// convolution's matrix Q (Section 4.1, Section 4) when more than four channels rule out the cofactor formulas.
#pragma once

namespace invconv {

// Q^-1 and log|det Q| by ONE wave: in-place Gauss-Jordan with partial pivoting, no barrier anywhere.  Rows never
// move: the pivot of column `col` is the largest entry of that column among the rows that have not been a pivot
// row yet, and own[col] remembers which row that was.  That is plain in-place elimination on the row-permuted
// matrix, so at the end row own[i] holds row i of the inverse with its columns in the same permutation:
//   Qinv[i][own[j]] = a[own[i]][j].
// Both forms write qinv[C][C] (LDS, doubles) and return sum log|pivot| in every lane.
__device__ __forceinline__ double readlane_f64(double v, int lane /* uniform */)
{
    const unsigned long long bits = __builtin_bit_cast(unsigned long long, v);
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)bits, lane);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(bits >> 32), lane);
    return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
}

// Pivot search: the candidates |entry| (or -1 for rows that may not be chosen) carry their row in the lowest seven
// bits of the mantissa, so one max over doubles finds value and row together (positive doubles order like their bit
// patterns; the seven bits only blur which of two nearly equal candidates wins).  Max over a row of 16 lanes by four
// DPP shifts, over the wave by two row broadcasts; ROWS16: all candidates sit in lanes 0 .. 15.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_mov_f64(double v)
{
    const unsigned long long bits = __builtin_bit_cast(unsigned long long, v);
    const int lo = (int)(unsigned)bits, hi = (int)(unsigned)(bits >> 32);
    const unsigned rlo = (unsigned)__builtin_amdgcn_update_dpp(lo, lo, CTRL, ROW_MASK, 0xf, false);
    const unsigned rhi = (unsigned)__builtin_amdgcn_update_dpp(hi, hi, CTRL, ROW_MASK, 0xf, false);
    return __builtin_bit_cast(double, ((unsigned long long)rhi << 32) | rlo);
}

template <bool ROWS16>
__device__ __forceinline__ int wave_pivot_row(double cand, int row)
{
    double key = cand;
    if (cand >= 0.0) {
        const unsigned long long bits = __builtin_bit_cast(unsigned long long, cand);
        key = __builtin_bit_cast(double, (bits & ~0x7full) | (unsigned long long)(127 - (row & 127)));
    }
    key = fmax(key, dpp_mov_f64<0x111, 0xf>(key));      // row_shr:1 (lanes without a source keep their own value)
    key = fmax(key, dpp_mov_f64<0x112, 0xf>(key));      // row_shr:2
    key = fmax(key, dpp_mov_f64<0x114, 0xf>(key));      // row_shr:4
    key = fmax(key, dpp_mov_f64<0x118, 0xf>(key));      // row_shr:8: lane 15 of a row holds the row's maximum
    if (!ROWS16) {
        key = fmax(key, dpp_mov_f64<0x142, 0xa>(key));  // row_bcast:15 into rows 1 and 3
        key = fmax(key, dpp_mov_f64<0x143, 0xc>(key));  // row_bcast:31 into rows 2 and 3: lane 63 holds the maximum
    }
    const double top = readlane_f64(key, ROWS16 ? 15 : 63);
    return 127 - (int)(__builtin_bit_cast(unsigned long long, top) & 0x7full);
}

// C <= 16: lane r holds row r in registers; every index below is a compile-time constant.
__device__ __forceinline__ double flow_invert_regs(const float *__restrict__ Q, int C, double *qinv)
{
    constexpr int N = 16;
    const int lane = threadIdx.x & 63;
    const bool mine = lane < C;
    double row[N], pivs[N];
#pragma unroll
    for (int c = 0; c < N; ++c)
        row[c] = (mine && c < C) ? (double)Q[lane * C + c] : 0.0;
    int own[N];
    bool used = !mine;
    int mycol = 0;
#pragma unroll
    for (int col = 0; col < N; ++col) {
        pivs[col] = 1.0;
        own[col] = 0;
        if (col < C) {
            const int p = wave_pivot_row<true>(used ? -1.0 : fabs(row[col]), lane);
            own[col] = p;
            double prow[N];
#pragma unroll
            for (int c = 0; c < N; ++c)
                prow[c] = readlane_f64(row[c], p);
            const double piv = prow[col], inv = 1.0 / piv;
            pivs[col] = piv;
#pragma unroll
            for (int c = 0; c < N; ++c)
                prow[c] = c == col ? inv : prow[c] * inv;
            const double f = row[col];
            if (lane == p) {
                used = true;
                mycol = col;
            }
#pragma unroll
            for (int c = 0; c < N; ++c) {
                const double upd = c == col ? -f * inv : row[c] - f * prow[c];
                row[c] = lane == p ? prow[c] : upd;
            }
        }
    }
    if (mine) {
#pragma unroll
        for (int j = 0; j < N; ++j)
            if (j < C)
                qinv[mycol * C + own[j]] = row[j];
    }
    // the logarithms of the pivots, one per lane, at the end (a double logarithm is a long routine)
    double pv = 1.0;
#pragma unroll
    for (int j = 0; j < N; ++j)
        pv = lane == j ? pivs[j] : pv;
    double la = log(fabs(pv));
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1)
        la += __shfl_xor(la, m, 64);
    return la;
}

}  // namespace invconv
