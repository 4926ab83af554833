// Shared device helpers of the inverse-convolution kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace invconv {

// Both triangular solves run the same code.  The transposed solve
// dL/dy = M^{-T} dL/dx (Eq. 2, Theorem 1) is the forward substitution of
// Section 3 applied in mirrored coordinates r' = H-1-r, c' = W-1-c,
// ch' = C-1-ch with the kernel w'[o'][i'][a][b] = w[C-1-i'][C-1-o'][a][b]:
// mirroring turns "depends on pixels below/right and channels above" into
// "depends on pixels above/left and channels below".  DIR = 0 is the plain
// (forward) orientation, DIR = 1 the mirrored one.
template <int DIR>
__device__ __forceinline__ size_t gidx(int n, int ch, int r, int c, int C, int H, int W)
{
    if (DIR) {
        ch = C - 1 - ch;
        r = H - 1 - r;
        c = W - 1 - c;
    }
    return (((size_t)n * C + ch) * H + r) * W + c;
}

// Kernel entry in solve coordinates, with the current-pixel block's upper
// triangle read as zero whatever the array holds.
template <int DIR>
__device__ __forceinline__ float weff(const float *__restrict__ w, int C, int k, int o, int i, int a, int b)
{
    const int oo = DIR ? C - 1 - i : o;
    const int ii = DIR ? C - 1 - o : i;
    if (a == k - 1 && b == k - 1 && ii > oo)
        return 0.0f;
    return w[((oo * C + ii) * k + a) * k + b];
}

// log|det dx/dy| of one image (Section 4), -H W sum_c log|w[c][c][k-1][k-1]|, by one full wave: lane l takes
// channels l, l + 64, ..., fixed butterfly across the lanes (the arithmetic of the stand-alone log-determinant
// kernel, so both give the same bits).  For kernels that have a wave to spare while the others set up.
__device__ __forceinline__ void wave_logdet_any(const float *__restrict__ w, int C, int k, int H, int W,
                                                float *__restrict__ out)
{
    const int lane = threadIdx.x & 63;
    double s = 0.0;
    for (int c = lane; c < C; c += 64)
        s += log(fabs((double)w[((c * C + c) * k + (k - 1)) * k + (k - 1)]));
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1)
        s += __shfl_xor(s, m, 64);
    if (lane == 0)
        out[0] = (float)(-(double)H * (double)W * s);
}

// Weight preparation, done by every workgroup for itself (C*C*k*k is at most
// a few thousand entries).  With L the lower-triangular current-pixel block,
//   x_p = L^{-1} ( y_p - sum_{tap != current} W_tap x_{p-tap} )
// so with Linv = L^{-1} and Cf_tap = Linv * W_tap the channels of one pixel no
// longer depend on each other:
//   x_p = Linv y_p - sum_tap Cf_tap x_{p-tap}.
// Outputs (LDS): sLinv[C][C]; sCf[k*k][C][C] indexed by tp = da*k+db where
// (da,db) = (k-1-a, k-1-b) is how far up/left the tap reaches (tp = 0 unused,
// zero filled).  sL is C*C floats of scratch and sW k*k*C*C floats of scratch
// (the oriented, masked kernel as [tp][o][i], read from global memory once).
// Ends with a barrier.
// CT = C when it is known at compile time (the folded taps then come from one forward substitution per column, in
// registers), 0 otherwise (staged copy, inverse, products).
template <int DIR, int CT = 0>
__device__ void fold_weights(const float *__restrict__ w, int C, int k,
                             float *sL, float *sLinv, float *sCf, float *sW)
{
    const int tid = threadIdx.x, nt = blockDim.x;
    const int total = k * k * C * C;
    if constexpr (CT > 0) {
        // C known at compile time: one thread per column (tp, i) of the k*k blocks solves  L cf = W_tap[:, i]  by
        // forward substitution in registers (tp = 0: the column of the identity, which gives column i of Linv).
        // Every load of the first round - the thread's own column and its share of L - is in flight before the
        // first wait, so the preparation costs one memory round trip, a barrier and C (C + 1) / 2 multiply-adds
        // per thread; L is read from LDS at addresses common to all lanes.
        constexpr int N = CT;
        constexpr int LT = (N * N + 63) / 64;       // shares of L per thread (a workgroup has at least 64 threads)
        auto entry = [&](int tp, int o, int i) -> float {
            const int a = k - 1 - tp / k, b = k - 1 - tp % k;
            const int oo = DIR ? N - 1 - i : o, ii = DIR ? N - 1 - o : i;
            const float v = w[((oo * N + ii) * k + a) * k + b];
            return (tp == 0 && ii > oo) ? 0.0f : v;     // the current-pixel block's upper triangle reads as zero
        };
        const int ncol = k * k * N;
        float col[N], lsh[LT];
        auto load_col = [&](int c) {
            const int cc = c < ncol ? c : ncol - 1;
            const int tp = cc / N, i = cc % N;
#pragma unroll
            for (int o = 0; o < N; ++o)
                col[o] = tp == 0 ? (o == i ? 1.0f : 0.0f) : entry(tp, o, i);
        };
#pragma unroll
        for (int u = 0; u < LT; ++u) {
            const int e = tid + u * nt;
            const int ec = e < N * N ? e : N * N - 1;
            lsh[u] = entry(0, ec / N, ec % N);
        }
        load_col(tid);
#pragma unroll
        for (int u = 0; u < LT; ++u) {
            const int e = tid + u * nt;
            if (e < N * N)
                sL[e] = lsh[u];
        }
        __syncthreads();
        for (int c = tid; c < ncol; c += nt) {
            if (c != tid)
                load_col(c);
            const int tp = c / N, i = c % N;
            float cf[N], rd[N];
#pragma unroll
            for (int o = 0; o < N; ++o)
                rd[o] = 1.0f / sL[o * N + o];
#pragma unroll
            for (int o = 0; o < N; ++o) {
                float acc = col[o];
#pragma unroll
                for (int m = 0; m < o; ++m)
                    acc -= sL[o * N + m] * cf[m];
                cf[o] = acc * rd[o];
            }
#pragma unroll
            for (int o = 0; o < N; ++o) {
                if (tp == 0)
                    sLinv[o * N + i] = cf[o];
                sCf[(tp * N + o) * N + i] = tp == 0 ? 0.0f : cf[o];
            }
        }
        __syncthreads();
        return;
    }
    // the kernel is read four entries per thread at a time (addresses clamped, no branch around a load),
    // so that the whole staging costs about one memory latency
    for (int base = tid; base < total; base += 4 * nt) {
        float val[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int raw = base + u * nt;
            const int idx = raw < total ? raw : total - 1;
            const int i = idx % C, o = (idx / C) % C, tp = idx / (C * C);
            const int a = k - 1 - tp / k, b = k - 1 - tp % k;
            const int oo = DIR ? C - 1 - i : o, ii = DIR ? C - 1 - o : i;
            const float v = w[((oo * C + ii) * k + a) * k + b];
            val[u] = (tp == 0 && ii > oo) ? 0.0f : v;       // the current-pixel block's upper triangle reads as zero
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = base + u * nt;
            if (idx < total) {
                sW[idx] = val[u];
                if (idx < C * C)
                    sL[idx] = val[u];       // tp == 0: idx = o * C + i
            }
        }
    }
    __syncthreads();
    if (tid < C) {
        const int j = tid;
        for (int o = 0; o < j; ++o)
            sLinv[o * C + j] = 0.0f;
        sLinv[j * C + j] = 1.0f / sL[j * C + j];
        for (int o = j + 1; o < C; ++o) {
            float s = 0.0f;
            for (int m = j; m < o; ++m)
                s += sL[o * C + m] * sLinv[m * C + j];
            sLinv[o * C + j] = -s / sL[o * C + o];
        }
    }
    __syncthreads();
    for (int idx = tid; idx < total; idx += nt) {
        const int i = idx % C, o = (idx / C) % C, tp = idx / (C * C);
        float s = 0.0f;
        if (tp != 0) {
            const float *li = sLinv + o * C;
            const float *wt = sW + tp * C * C + i;
            for (int j = 0; j <= o; ++j)
                s += li[j] * wt[j * C];
        }
        sCf[idx] = s;
    }
    __syncthreads();
}

// The earlier form of the preparation for a compile-time C: the kernel staged in LDS (sW), Linv by one thread per
// column, the products Linv W_tap from LDS.  Three rounds instead of one, but it keeps fewer values per thread: in
// the pipelined stack kernel (sixteen waves of 128 registers) it measures 22 us less per launch than the
// substitution form above, and a launch of that kernel prepares its weights once in half a millisecond.
template <int DIR, int CT = 0>
__device__ void fold_weights_staged(const float *__restrict__ w, int C, int k,
                             float *sL, float *sLinv, float *sCf, float *sW)
{
    const int tid = threadIdx.x, nt = blockDim.x;
    const int total = k * k * C * C;
    // the kernel is read four entries per thread at a time (addresses clamped, no branch around a load),
    // so that the whole staging costs about one memory latency
    for (int base = tid; base < total; base += 4 * nt) {
        float val[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int raw = base + u * nt;
            const int idx = raw < total ? raw : total - 1;
            const int i = idx % C, o = (idx / C) % C, tp = idx / (C * C);
            const int a = k - 1 - tp / k, b = k - 1 - tp % k;
            const int oo = DIR ? C - 1 - i : o, ii = DIR ? C - 1 - o : i;
            const float v = w[((oo * C + ii) * k + a) * k + b];
            val[u] = (tp == 0 && ii > oo) ? 0.0f : v;       // the current-pixel block's upper triangle reads as zero
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = base + u * nt;
            if (idx < total) {
                sW[idx] = val[u];
                if (idx < C * C)
                    sL[idx] = val[u];       // tp == 0: idx = o * C + i
            }
        }
    }
    __syncthreads();
    if (CT > 0) {
        // column j of Linv by forward substitution in registers: the needed part of L and the reciprocals
        // of its diagonal are fetched first, so the chain over o is multiply-adds only (entries above the
        // diagonal stay zero, so the inner sum needs no lower bound)
        if (tid < CT) {
            const int j = tid;
            constexpr int N = CT > 0 ? CT : 1;
            float Lr[N][N], rd[N], lv[N];
#pragma unroll
            for (int o = 0; o < N; ++o)
#pragma unroll
                for (int m = 0; m <= o; ++m)
                    Lr[o][m] = sL[o * N + m];
#pragma unroll
            for (int o = 0; o < N; ++o)
                rd[o] = 1.0f / Lr[o][o];
#pragma unroll
            for (int o = 0; o < N; ++o) {
                float acc = 0.0f;
#pragma unroll
                for (int m = 0; m < o; ++m)
                    acc += Lr[o][m] * lv[m];
                lv[o] = (o == j) ? rd[o] : (o > j ? -acc * rd[o] : 0.0f);
                sLinv[o * N + j] = lv[o];
            }
        }
    } else if (tid < C) {
        const int j = tid;
        for (int o = 0; o < j; ++o)
            sLinv[o * C + j] = 0.0f;
        sLinv[j * C + j] = 1.0f / sL[j * C + j];
        for (int o = j + 1; o < C; ++o) {
            float s = 0.0f;
            for (int m = j; m < o; ++m)
                s += sL[o * C + m] * sLinv[m * C + j];
            sLinv[o * C + j] = -s / sL[o * C + o];
        }
    }
    __syncthreads();
    if (CT > 0) {
        // two outputs per trip, so that the LDS reads of one overlap the arithmetic of the other
        // (entries of Linv above the diagonal are zero, so the full row may be used)
        for (int idx = tid; idx < total; idx += 2 * nt) {
            const int idx2 = idx + nt < total ? idx + nt : idx;
            const int i = idx % CT, o = (idx / CT) % CT, tp = idx / (CT * CT);
            const int i2 = idx2 % CT, o2 = (idx2 / CT) % CT, tp2 = idx2 / (CT * CT);
            const float *li = sLinv + o * CT, *wt = sW + tp * CT * CT + i;
            const float *li2 = sLinv + o2 * CT, *wt2 = sW + tp2 * CT * CT + i2;
            float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
            for (int j = 0; j < (CT > 0 ? CT : 1); ++j) {
                s1 += li[j] * wt[j * CT];
                s2 += li2[j] * wt2[j * CT];
            }
            sCf[idx] = tp != 0 ? s1 : 0.0f;
            if (idx + nt < total)
                sCf[idx2] = tp2 != 0 ? s2 : 0.0f;
        }
    } else {
        for (int idx = tid; idx < total; idx += nt) {
            const int i = idx % C, o = (idx / C) % C, tp = idx / (C * C);
            float s = 0.0f;
            if (tp != 0) {
                const float *li = sLinv + o * C;
                const float *wt = sW + tp * C * C + i;
                for (int j = 0; j <= o; ++j)
                    s += li[j] * wt[j * C];
            }
            sCf[idx] = s;
        }
    }
    __syncthreads();
}

// The same preparation for many channels, where a second k*k*C*C staging buffer would not fit LDS: the
// kernel entries are read from global memory where they are used (every entry C times, from L2).
// Outputs sL, sLinv (C*C each) and sCf (k*k*C*C) as above.  Ends with a barrier.
template <int DIR>
__device__ void fold_weights_lean(const float *__restrict__ w, int C, int k, float *sL, float *sLinv, float *sCf)
{
    const int tid = threadIdx.x, nt = blockDim.x;
    // oriented, masked entry (tp, o, i)
    auto entry = [&](int tp, int o, int i) -> float {
        const int a = k - 1 - tp / k, b = k - 1 - tp % k;
        const int oo = DIR ? C - 1 - i : o, ii = DIR ? C - 1 - o : i;
        const float v = w[((oo * C + ii) * k + a) * k + b];
        return (tp == 0 && ii > oo) ? 0.0f : v;
    };
    for (int idx = tid; idx < C * C; idx += nt)
        sL[idx] = entry(0, idx / C, idx % C);
    __syncthreads();
    if (tid < C) {
        const int j = tid;
        for (int o = 0; o < j; ++o)
            sLinv[o * C + j] = 0.0f;
        sLinv[j * C + j] = 1.0f / sL[j * C + j];
        for (int o = j + 1; o < C; ++o) {
            float s = 0.0f;
            for (int m = j; m < o; ++m)
                s += sL[o * C + m] * sLinv[m * C + j];
            sLinv[o * C + j] = -s / sL[o * C + o];
        }
    }
    __syncthreads();
    const int total = k * k * C * C;
    for (int idx = tid; idx < total; idx += nt) {
        const int i = idx % C, o = (idx / C) % C, tp = idx / (C * C);
        float s = 0.0f;
        if (tp != 0) {
            const float *li = sLinv + o * C;
            for (int j = 0; j <= o; ++j)
                s += li[j] * entry(tp, j, i);
        }
        sCf[idx] = s;
    }
    __syncthreads();
}

}  // namespace invconv
