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
// CT = C when it is known at compile time (loops then have fixed trip counts and
// their LDS reads pipeline), 0 otherwise.
template <int DIR, int CT = 0>
__device__ void fold_weights(const float *__restrict__ w, int C, int k,
                             float *sL, float *sLinv, float *sCf, float *sW)
{
    const int tid = threadIdx.x, nt = blockDim.x;
    const int total = k * k * C * C;
    for (int idx = tid; idx < total; idx += nt) {
        const int i = idx % C, o = (idx / C) % C, tp = idx / (C * C);
        const float val = weff<DIR>(w, C, k, o, i, k - 1 - tp / k, k - 1 - tp % k);
        sW[idx] = val;
        if (tp == 0)
            sL[o * C + i] = val;
    }
    __syncthreads();
    if (CT > 0) {
        // column j of Linv by forward substitution, kept in registers (all loops unrolled,
        // entries above the diagonal stay zero so the inner sum needs no lower bound)
        if (tid < CT) {
            const int j = tid;
            float lv[CT > 0 ? CT : 1];
#pragma unroll
            for (int o = 0; o < CT; ++o) {
                float s = 0.0f;
#pragma unroll
                for (int m = 0; m < o; ++m)
                    s += sL[o * CT + m] * lv[m];
                const float d = sL[o * CT + o];
                lv[o] = (o == j) ? 1.0f / d : (o > j ? -s / d : 0.0f);
                sLinv[o * CT + j] = lv[o];
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
    for (int idx = tid; idx < total; idx += nt) {
        const int i = idx % C, o = (idx / C) % C, tp = idx / (C * C);
        float s = 0.0f;
        if (tp != 0) {
            const float *li = sLinv + o * C;
            const float *wt = sW + tp * C * C + i;
            if (CT > 0) {
                // entries of Linv above the diagonal are zero, so the full row may be used
#pragma unroll
                for (int j = 0; j < CT; ++j)
                    s += li[j] * wt[j * CT];
            } else {
                for (int j = 0; j <= o; ++j)
                    s += li[j] * wt[j * C];
            }
        }
        sCf[idx] = s;
    }
    __syncthreads();
}

}  // namespace invconv
