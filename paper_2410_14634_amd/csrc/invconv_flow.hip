// One flow step around the inverse convolution (Section 4.1: Inv-Conv layer, Actnorm layer, 1 x 1
// convolution; log-determinants of Section 4):
//     x = invconv_w(y),   a = s * x + b (per channel),   z = Q a (per pixel)
// so z = A x + d with A = Q diag(s), d = Q b: the two neighbours are ONE affine channel map per pixel.
// Forward: only z is written.  Backward: x is recomputed as A^-1 (z - d), the upstream gradient enters the
// transposed solve as A^T dL/dz, and the neighbours' parameter gradients follow from two sums over batch and
// pixels,  M2[o][i] = sum dL/dz[o] x[i]  and  m1[o] = sum dL/dz[o]:
//     dL/dQ[o][i] = s[i] M2[o][i] + b[i] m1[o],  dL/ds[i] = sum_o Q[o][i] M2[o][i],  dL/db[i] = sum_o Q[o][i] m1[o].
// For few-channel images that fit LDS the whole step is fused around the single-wave solve (the image is in
// LDS anyway): forward and backward each read and write what the inverse convolution alone would.  Other
// shapes run the same arithmetic as separate passes.  gfx950 only.
#include "invconv_common.h"
#include "invconv_launch.h"
#include "invconv_small_mat.h"
#include "invconv_wave_inverse.h"
#include "invconv_wave_solve.h"

namespace invconv {

// ---------------------------------------------------------------------------
// Small matrices of a step, prepared once per call by one workgroup (double arithmetic):
//   A[o][i] = Q[o][i] s[i],  d[o] = sum_i Q[o][i] b[i],  Ainv = A^-1 = diag(1/s) Q^-1 (Gauss-Jordan with
//   partial pivoting, by one wave),  e = -Ainv d = -b/s,  QinvT = Q^-T (for the log-determinant's gradient), and
//   logdet = -H W sum log|w[c][c][k-1][k-1]| + H W sum log|s[c]| + H W log|det Q|   (one image).
// Layout (floats): A, d, Ainv, e, QinvT, logdet.  A singular Q gives inf / NaN, as a zero diagonal does.
// ---------------------------------------------------------------------------
__host__ __device__ constexpr int flow_off_d(int C) { return C * C; }
__host__ __device__ constexpr int flow_off_Ainv(int C) { return C * C + C; }
__host__ __device__ constexpr int flow_off_e(int C) { return 2 * C * C + C; }
__host__ __device__ constexpr int flow_off_QinvT(int C) { return 2 * C * C + 2 * C; }
__host__ __device__ constexpr int flow_off_logdet(int C) { return 3 * C * C + 2 * C; }
size_t flow_mats_floats(int C) { return (size_t)3 * C * C + 2 * C + 1; }

// Up to 128 channels, all waves of the workgroup: the matrix lives in `a` (row stride C + 1 doubles).  The first
// wave finds the pivot row of a column (lane l looks at rows l and l + 64), keeps a copy of the column (the
// factors) and scales the pivot row; after a barrier every wave eliminates its share of the COLUMNS from all rows
// (lane = row; a row's entries are consecutive addresses, four at a time); a second barrier ends the step.
__device__ __forceinline__ double flow_invert_lds(const float *__restrict__ Q, int C, double *a, double *fcol,
                                                  double *pivs, int *own, double *qinv)
{
    const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63, wave = tid >> 6, nw = nt >> 6, LD = C + 1;
    for (int e = tid; e < C * C; e += nt)
        a[(e / C) * LD + e % C] = (double)Q[e];
    __syncthreads();
    const int cw = ((C + nw - 1) / nw + 3) & ~3;        // columns per wave, whole groups of four
    const int c_lo = wave * cw, c_hi = c_lo + cw < C ? c_lo + cw : C;
    unsigned used = 0;          // (first wave) bit t: row lane + 64 t has been a pivot row
    for (int col = 0; col < C; ++col) {
        if (wave == 0) {
            double best = -1.0;
            int br = lane;
            for (int r = lane, t = 0; r < C; r += 64, ++t) {
                const double v = a[r * LD + col];
                fcol[r] = v;
                const double cand = (used >> t) & 1 ? -1.0 : fabs(v);
                if (cand > best) {
                    best = cand;
                    br = r;
                }
            }
            const int p = wave_pivot_row<false>(best, br);
            if ((p & 63) == lane)
                used |= 1u << (p >> 6);
            const double piv = a[p * LD + col], inv = 1.0 / piv;
            if (lane == 0) {
                own[col] = p;
                pivs[col] = piv;
            }
            for (int c = lane; c < C; c += 64)
                a[p * LD + c] = c == col ? inv : a[p * LD + c] * inv;
        }
        __syncthreads();
        const int p = own[col];
        const double inv = a[p * LD + col];
        const double *ap = a + p * LD;
        for (int r = lane; r < C; r += 64) {
            if (r == p)
                continue;
            double *ar = a + r * LD;
            const double f = fcol[r];
            for (int c0 = c_lo; c0 < c_hi; c0 += 4) {       // (the pad entry ar[C] is scratch for the columns past the end)
                double pv[4], rv[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int c = c0 + u < c_hi ? c0 + u : C;
                    pv[u] = ap[c];
                    rv[u] = ar[c];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int c = c0 + u < c_hi ? c0 + u : C;
                    ar[c] = c == col ? -f * inv : rv[u] - f * pv[u];
                }
            }
        }
        __syncthreads();
    }
    for (int e = tid; e < C * C; e += nt) {
        const int i = e / C, j = e % C;
        qinv[i * C + own[j]] = a[own[i] * LD + j];
    }
    double la = 0.0;            // the pivots' logarithms at the end, one column per lane and trip (first wave)
    if (wave == 0) {
        for (int c = lane; c < C; c += 64)
            la += log(fabs(pivs[c]));
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1)
            la += __shfl_xor(la, m, 64);
    }
    return la;
}

// (WIDE: more than 16 channels, sixteen waves share the elimination)
template <bool WIDE>
__global__ __launch_bounds__(WIDE ? 1024 : 256) void k_flow_prep(const float *__restrict__ w, const float *__restrict__ s,
                                                  const float *__restrict__ b, const float *__restrict__ Q,
                                                  float *__restrict__ mats, float *__restrict__ logdet_out, int C,
                                                  int H, int W, int k)
{
    extern __shared__ double sm[];
    double *qinv = sm;                      // [C][C]
    double *work = sm + C * C;              // [C][C + 1] (more than 16 channels)
    double *fcol = work + C * (C + 1);      // [C]
    double *pivs = fcol + C;                // [C]
    int *own = reinterpret_cast<int *>(pivs + C);       // [C]
    __shared__ double s_logabs;
    const int tid = threadIdx.x, nt = blockDim.x;
    double la = 0.0;
    if constexpr (WIDE)
        la = flow_invert_lds(Q, C, work, fcol, pivs, own, qinv);
    else if (tid < 64)
        la = flow_invert_regs(Q, C, qinv);
    if (tid == 0)
        s_logabs = la;
    __syncthreads();
    for (int e = tid; e < C * C; e += nt) {
        const int o = e / C, i = e % C;
        mats[e] = Q[e] * s[i];                                                          // A[o][i]
        mats[flow_off_Ainv(C) + e] = (float)(qinv[o * C + i] / (double)s[o]);           // Ainv[o][i] (row o of Q^-1 over s[o])
        mats[flow_off_QinvT(C) + e] = (float)qinv[i * C + o];                           // QinvT[o][i] = Qinv[i][o]
    }
    for (int o = tid; o < C; o += nt) {
        double acc = 0.0;
        for (int i = 0; i < C; ++i)
            acc += (double)Q[o * C + i] * (double)b[i];
        mats[flow_off_d(C) + o] = (float)acc;
        mats[flow_off_e(C) + o] = -b[o] / s[o];
    }
    if (tid < 64) {     // one channel per lane and trip: the logarithms are the long part
        double acc = 0.0;
        for (int c = tid; c < C; c += 64)
            acc += log(fabs((double)s[c])) - log(fabs((double)w[((c * C + c) * k + (k - 1)) * k + (k - 1)]));
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1)
            acc += __shfl_xor(acc, m, 64);
        if (tid == 0) {
            const float ld = (float)((double)H * (double)W * (acc + s_logabs));
            mats[flow_off_logdet(C)] = ld;
            if (logdet_out)
                logdet_out[0] = ld;
        }
    }
}

// ---------------------------------------------------------------------------
// Separate pass: out[n][o][p] = add[o] + sum_i M[o][i] in[n][i][p]  (TR: M[i][o] instead), one thread per
// four consecutive pixels when the planes allow 16-byte accesses, else per pixel.  `out` may be `in`: a
// thread reads all its inputs before it writes.  CT = C (1-4, 8, 12, 16: the inputs stay in registers).
// ---------------------------------------------------------------------------
template <int CT, int VEC, bool TR>
__global__ __launch_bounds__(256) void k_flow_affine(const float *in, const float *__restrict__ M,
                                                    const float *__restrict__ add, float *out, int C, int HW,
                                                    long long total /* B * HW / VEC */)
{
    typedef float vec_t __attribute__((ext_vector_type(VEC)));
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= total)
        return;
    const int per = HW / VEC;
    const long long n = t / per;
    const int q = (int)(t % per);
    const vec_t *src = reinterpret_cast<const vec_t *>(in + (size_t)n * C * HW) + q;
    vec_t *dst = reinterpret_cast<vec_t *>(out + (size_t)n * C * HW) + q;
    static_assert(CT > 0, "channel counts without a register-resident form take k_flow_affine_blocked");
    {
        vec_t xin[CT];
#pragma unroll
        for (int i = 0; i < CT; ++i)
            xin[i] = src[(size_t)i * per];
#pragma unroll
        for (int o = 0; o < CT; ++o) {
            const float a0 = add ? add[o] : 0.0f;
            vec_t acc;
#pragma unroll
            for (int u = 0; u < VEC; ++u)
                acc[u] = a0;
#pragma unroll
            for (int i = 0; i < CT; ++i)
                acc += (TR ? M[i * CT + o] : M[o * CT + i]) * xin[i];
            dst[(size_t)o * per] = acc;
        }
    }
}

// Other channel counts (5-7, 9-11, 13-15 and everything above 16): a thread forms OT = 8 output channels of its
// pixels (blockIdx.y selects which eight), reading every input channel once; the matrix entries are the same
// address for all lanes.  A read is repeated by the C / 8 threads of a pixel (cache hits); `out` must not alias
// `in`.
template <int VEC, bool TR>
__global__ __launch_bounds__(256) void k_flow_affine_blocked(const float *__restrict__ in, const float *__restrict__ M,
                                                            const float *__restrict__ add, float *__restrict__ out,
                                                            int C, int HW, long long total /* B * HW / VEC */)
{
    constexpr int OT = 8;
    typedef float vec_t __attribute__((ext_vector_type(VEC)));
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= total)
        return;
    const int per = HW / VEC;
    const long long n = t / per;
    const int q = (int)(t % per);
    const int o0 = blockIdx.y * OT;
    const vec_t *src = reinterpret_cast<const vec_t *>(in + (size_t)n * C * HW) + q;
    vec_t *dst = reinterpret_cast<vec_t *>(out + (size_t)n * C * HW) + q;
    vec_t acc[OT];
    int orow[OT];       // clamped output channel: rows past the end repeat the last one and are not stored
#pragma unroll
    for (int u = 0; u < OT; ++u) {
        orow[u] = o0 + u < C ? o0 + u : C - 1;
        const float a0 = add ? add[orow[u]] : 0.0f;
#pragma unroll
        for (int e = 0; e < VEC; ++e)
            acc[u][e] = a0;
    }
    for (int i0 = 0; i0 < C; i0 += 4) {       // four input channels in flight
        vec_t xin[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            xin[j] = src[(size_t)(i0 + j < C ? i0 + j : C - 1) * per];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (i0 + j < C) {
#pragma unroll
                for (int u = 0; u < OT; ++u)
                    acc[u] += (TR ? M[(i0 + j) * C + orow[u]] : M[orow[u] * C + i0 + j]) * xin[j];
            }
        }
    }
#pragma unroll
    for (int u = 0; u < OT; ++u)
        if (o0 + u < C)
            dst[(size_t)(o0 + u) * per] = acc[u];
}

template <int CT, bool TR>
static void launch_affine_ct(const float *in, const float *M, const float *add, float *out, int B, int C, int HW,
                             hipStream_t stream)
{
    const bool vec = (HW % 4) == 0 && ((((size_t)in) | ((size_t)out)) & 15) == 0;
    const long long total = (long long)B * HW / (vec ? 4 : 1);
    const unsigned grid = (unsigned)((total + 255) / 256);
    if constexpr (CT == 0) {
        const dim3 g2(grid, (unsigned)((C + 7) / 8));
        if (vec)
            hipLaunchKernelGGL((k_flow_affine_blocked<4, TR>), g2, dim3(256), 0, stream, in, M, add, out, C, HW, total);
        else
            hipLaunchKernelGGL((k_flow_affine_blocked<1, TR>), g2, dim3(256), 0, stream, in, M, add, out, C, HW, total);
    } else if (vec) {
        hipLaunchKernelGGL((k_flow_affine<CT, 4, TR>), dim3(grid), dim3(256), 0, stream, in, M, add, out, C, HW, total);
    } else {
        hipLaunchKernelGGL((k_flow_affine<CT, 1, TR>), dim3(grid), dim3(256), 0, stream, in, M, add, out, C, HW, total);
    }
}

template <bool TR>
static int launch_affine(const float *in, const float *M, const float *add, float *out, int B, int C, int HW,
                         hipStream_t stream)
{
    switch (C) {
    case 1: launch_affine_ct<1, TR>(in, M, add, out, B, C, HW, stream); break;
    case 2: launch_affine_ct<2, TR>(in, M, add, out, B, C, HW, stream); break;
    case 3: launch_affine_ct<3, TR>(in, M, add, out, B, C, HW, stream); break;
    case 4: launch_affine_ct<4, TR>(in, M, add, out, B, C, HW, stream); break;
    case 8: launch_affine_ct<8, TR>(in, M, add, out, B, C, HW, stream); break;
    case 12: launch_affine_ct<12, TR>(in, M, add, out, B, C, HW, stream); break;
    case 16: launch_affine_ct<16, TR>(in, M, add, out, B, C, HW, stream); break;
    default:
        if (in == out)
            return INVCONV_ERR_ALIAS;
        launch_affine_ct<0, TR>(in, M, add, out, B, C, HW, stream);
        break;
    }
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

// ---------------------------------------------------------------------------
// Separate pass: partial sums of M2[o][i] = sum gz[o] x[i] and m1[o] = sum gz[o] over one chunk of pixels of
// one image; row layout [C*C | C].  Fixed partition, fixed order inside a thread: deterministic.
// ---------------------------------------------------------------------------
constexpr int kFlowStatPix = 128;       // pixels per chunk

__global__ __launch_bounds__(256) void k_flow_stats(const float *__restrict__ gz, const float *__restrict__ x,
                                                   float *__restrict__ rows, int C, int HW, int chunks)
{
    extern __shared__ float fsm[];
    float *sg = fsm;                        // [C][kFlowStatPix]
    float *sx = fsm + C * kFlowStatPix;     // [C][kFlowStatPix]
    const int n = blockIdx.x / chunks, ch = blockIdx.x % chunks;
    const int p0 = ch * kFlowStatPix;
    const int np = HW - p0 < kFlowStatPix ? HW - p0 : kFlowStatPix;
    const int tid = threadIdx.x;
    for (int idx = tid; idx < C * kFlowStatPix; idx += 256) {
        const int c = idx / kFlowStatPix, p = idx % kFlowStatPix;
        const bool ok = p < np;
        const size_t src = ((size_t)n * C + c) * HW + p0 + (ok ? p : 0);
        const float gv = gz[src], xv = x[src];
        sg[idx] = ok ? gv : 0.0f;
        sx[idx] = ok ? xv : 0.0f;
    }
    __syncthreads();
    const int E = C * C + C;
    float *row = rows + (size_t)blockIdx.x * E;
    for (int e = tid; e < E; e += 256) {
        float acc = 0.0f;
        if (e < C * C) {
            const float *pg = sg + (e / C) * kFlowStatPix, *px = sx + (e % C) * kFlowStatPix;
            for (int p = 0; p < kFlowStatPix; ++p)
                acc += pg[p] * px[p];
        } else {
            const float *pg = sg + (e - C * C) * kFlowStatPix;
            for (int p = 0; p < kFlowStatPix; ++p)
                acc += pg[p];
        }
        row[e] = acc;
    }
}

// ---------------------------------------------------------------------------
// Separate-pass backward, first launch: ONE pass over z and dL/dz of a chunk of 128 pixels of one image gives
//   x = A^-1 z - b/s  and  g = A^T dL/dz  (written out: the inputs of the inverse convolution's backward pass)
// and, from the tiles while they are in LDS, the chunk's partial sums of M2 and m1 (row layout [C*C | C] as above).
// It replaces two passes of the channel map and a pass of sums that read x and dL/dz again.  Tile rows are
// 129 floats apart: the threads of the sums walk rows that start in different banks.
// ---------------------------------------------------------------------------
constexpr int kFlowStatStride = kFlowStatPix + 1;

__global__ __launch_bounds__(256) void k_flow_bwd_maps(const float *__restrict__ z, const float *__restrict__ gz,
                                                      const float *__restrict__ mats, float *__restrict__ x,
                                                      float *__restrict__ g, float *__restrict__ rows, int C, int HW,
                                                      int chunks)
{
    extern __shared__ float fsm[];
    constexpr int PS = kFlowStatStride;
    float *sz = fsm;                        // [C][PS]
    float *sg = sz + C * PS;                // [C][PS]
    float *sx = sg + C * PS;                // [C][PS]
    float *sA = sx + C * PS;                // [C][C]  A
    float *sAi = sA + C * C;                // [C][C]  A^-1
    float *se = sAi + C * C;                // [C]     -b/s
    const int n = blockIdx.x / chunks, ch = blockIdx.x % chunks;
    const int p0 = ch * kFlowStatPix;
    const int np = HW - p0 < kFlowStatPix ? HW - p0 : kFlowStatPix;
    const int tid = threadIdx.x;
    for (int idx = tid; idx < C * kFlowStatPix; idx += 256) {
        const int c = idx / kFlowStatPix, p = idx % kFlowStatPix;
        const bool ok = p < np;
        const size_t src = ((size_t)n * C + c) * HW + p0 + (ok ? p : 0);
        const float zv = z[src], gv = gz[src];
        sz[c * PS + p] = ok ? zv : 0.0f;
        sg[c * PS + p] = ok ? gv : 0.0f;
    }
    for (int idx = tid; idx < C * C; idx += 256) {
        sA[idx] = mats[idx];
        sAi[idx] = mats[flow_off_Ainv(C) + idx];
    }
    for (int idx = tid; idx < C; idx += 256)
        se[idx] = mats[flow_off_e(C) + idx];
    __syncthreads();
    {
        // thread = (pixel p, half h): channels h, h + 2, ... of that pixel (the channel is the same for a whole wave)
        const int p = tid & (kFlowStatPix - 1), h = tid >> 7;
        const bool ok = p < np;
        for (int i = h; i < C; i += 2) {
            float xa = se[i], ga = 0.0f;
            for (int o = 0; o < C; ++o) {
                xa += sAi[i * C + o] * sz[o * PS + p];
                ga += sA[o * C + i] * sg[o * PS + p];
            }
            sx[i * PS + p] = ok ? xa : 0.0f;        // pixels past the end add nothing to the sums
            if (ok) {
                const size_t dst = ((size_t)n * C + i) * HW + p0 + p;
                x[dst] = xa;
                g[dst] = ga;
            }
        }
    }
    __syncthreads();
    const int E = C * C + C;
    float *row = rows + (size_t)blockIdx.x * E;
    for (int e = tid; e < E; e += 256) {
        float acc = 0.0f;
        if (e < C * C) {
            const float *pg = sg + (e / C) * PS, *px = sx + (e % C) * PS;
            for (int p = 0; p < kFlowStatPix; ++p)
                acc += pg[p] * px[p];
        } else {
            const float *pg = sg + (e - C * C) * PS;
            for (int p = 0; p < kFlowStatPix; ++p)
                acc += pg[p];
        }
        row[e] = acc;
    }
}

// m1 partial sums: one workgroup per (image, channel) plane adds its H*W values of dL/dz in a fixed order
// (thread t takes elements t, t + 256, ...; then a fixed tree over the 256 threads).  out[n*C + c].
__global__ __launch_bounds__(256) void k_flow_plane_sum(const float *__restrict__ gz, float *__restrict__ out, int HW)
{
    __shared__ float red[256];
    const float *p = gz + (size_t)blockIdx.x * HW;
    float acc = 0.0f;
    for (int i = threadIdx.x; i < HW; i += 256)
        acc += p[i];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int half = 128; half >= 1; half >>= 1) {
        if ((int)threadIdx.x < half)
            red[threadIdx.x] += red[threadIdx.x + half];
        __syncthreads();
    }
    if (threadIdx.x == 0)
        out[blockIdx.x] = red[0];
}

// Sum of `nrows` rows of `E` floats (row stride `stride`) in index order, double accumulator: wave v of a
// workgroup adds rows v, v + NW, ..., then the waves are added in order.  out[e] = the sum as float.
template <int NW>
__global__ __launch_bounds__(64 * NW) void k_rows_sum(const float *__restrict__ rows, int nrows, int stride, int E,
                                                     float *__restrict__ out)
{
    __shared__ double swave[NW][64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int e = blockIdx.x * 64 + lane;
    double acc = 0.0;
    if (e < E) {
        int p = wave;
        for (; p + 7 * NW < nrows; p += 8 * NW) {
            float a[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                a[u] = rows[(size_t)(p + NW * u) * stride + e];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                acc += (double)a[u];
        }
        if (p < nrows) {        // the last rows, loaded together (clamped addresses, rows past the end count as zero)
            float a[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int r = p + NW * u;
                a[u] = rows[(size_t)(r < nrows ? r : nrows - 1) * stride + e];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                acc += p + NW * u < nrows ? (double)a[u] : 0.0;
        }
    }
    swave[wave][lane] = acc;
    __syncthreads();
    if (wave == 0 && e < E) {
        double total = swave[0][lane];
#pragma unroll
        for (int v = 1; v < NW; ++v)
            total += swave[v][lane];
        out[e] = (float)total;
    }
}

// ---------------------------------------------------------------------------
// Last kernel of a backward call.  `sums` holds the summed rows: [P] un-negated dL/dw sums when the fused
// kernel produced them (have_dw), then [C*C] M2 and [C] m1.  Writes
//   dLdw (only with have_dw) = -sums, 0 at masked entries;
//   dLdQ, dLds, dLdb from M2, m1 (formulas above);
// and adds lw times the gradient of the step's log-determinant (Section 4; closed forms):
//   dLdw[c][c][k-1][k-1] -= lw H W / w[c][c][k-1][k-1],  dLds[c] += lw H W / s[c],  dLdQ += lw H W Q^-T.
// ---------------------------------------------------------------------------
// (sums and QinvT = Q^-T may live in LDS or in global memory; nt threads)
__device__ __forceinline__ void flow_finish_body(const float *sums, int have_dw, const float *__restrict__ w,
                                                 const float *__restrict__ s, const float *__restrict__ b,
                                                 const float *__restrict__ Q, const float *QinvT,
                                                 float *__restrict__ dLdw, float *__restrict__ dLds,
                                                 float *__restrict__ dLdb, float *__restrict__ dLdQ, float lw, int C,
                                                 int H, int W, int k, int tid, int nt)
{
    const int P = C * C * k * k;
    const float hw = (float)H * (float)W;
    const float *M2 = sums + (have_dw ? P : 0), *m1 = M2 + C * C;
    if (have_dw) {
        for (int e = tid; e < P; e += nt) {
            const int bb = e % k, a = (e / k) % k, i = (e / (k * k)) % C, o = e / (k * k * C);
            const bool centre = a == k - 1 && bb == k - 1;
            float v = (centre && i > o) ? 0.0f : -sums[e];
            if (centre && i == o && lw != 0.0f)
                v -= lw * hw / w[e];
            dLdw[e] = v;
        }
    } else if (lw != 0.0f) {
        // dL/dw is already there: only the C diagonal entries of the current-pixel block take the log-determinant's term
        for (int c = tid; c < C; c += nt) {
            const int e = ((c * C + c) * k + (k - 1)) * k + (k - 1);
            dLdw[e] -= lw * hw / w[e];
        }
    }
    for (int e = tid; e < C * C; e += nt) {
        const int o = e / C, i = e % C;
        float v = s[i] * M2[e] + b[i] * m1[o];
        if (lw != 0.0f)
            v += lw * hw * QinvT[e];
        dLdQ[e] = v;
    }
    for (int i = tid; i < C; i += nt) {
        float vs = 0.0f, vb = 0.0f;
        for (int o = 0; o < C; ++o) {
            vs += Q[o * C + i] * M2[o * C + i];
            vb += Q[o * C + i] * m1[o];
        }
        if (lw != 0.0f)
            vs += lw * hw / s[i];
        dLds[i] = vs;
        dLdb[i] = vb;
    }
}

__global__ __launch_bounds__(256) void k_flow_finish(const float *__restrict__ sums, int have_dw,
                                                    const float *__restrict__ w, const float *__restrict__ s,
                                                    const float *__restrict__ b, const float *__restrict__ Q,
                                                    const float *__restrict__ mats, float *__restrict__ dLdw,
                                                    float *__restrict__ dLds, float *__restrict__ dLdb,
                                                    float *__restrict__ dLdQ, float lw, int C, int H, int W, int k)
{
    flow_finish_body(sums, have_dw, w, s, b, Q, mats + flow_off_QinvT(C), dLdw, dLds, dLdb, dLdQ, lw, C, H, W, k,
                     threadIdx.x, 256);
}

// The same last step for few channels and at most a few hundred images, straight from the per-image rows
// [P | C*C | C] of the fused backward kernel: sixteen waves add the rows in a fixed order (wave v rows v, v + 16,
// ..., double accumulators, then the waves in order), Q^-T comes from cofactors, no other launch is needed.
template <int C>
__global__ __launch_bounds__(1024) void k_flow_finish_rows(const float *__restrict__ rows, int nrows,
                                                          const float *__restrict__ w, const float *__restrict__ s,
                                                          const float *__restrict__ b, const float *__restrict__ Q,
                                                          float *__restrict__ dLdw, float *__restrict__ dLds,
                                                          float *__restrict__ dLdb, float *__restrict__ dLdQ, float lw,
                                                          int H, int W, int k)
{
    constexpr int NW = 16, EMAX = C * C * 3 * 3 + C * C + C, NCH = (EMAX + 63) / 64;
    __shared__ double swave[NW][NCH * 64];
    __shared__ float ssum[NCH * 64];
    __shared__ float sQinvT[C * C];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int E = C * C * k * k + C * C + C;       // k = 3: E = EMAX
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
        const int e = ch * 64 + lane;
        double acc = 0.0;
        if (e < E) {
            for (int p = wave; p < nrows; p += 8 * NW) {        // eight rows in flight (clamped addresses)
                float a[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int r = p + NW * u;
                    a[u] = rows[(size_t)(r < nrows ? r : nrows - 1) * E + e];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    acc += p + NW * u < nrows ? (double)a[u] : 0.0;
            }
        }
        swave[wave][e] = acc;
    }
    if (tid < C * C) {
        double q[C][C], qi[C][C];
#pragma unroll
        for (int o = 0; o < C; ++o)
#pragma unroll
            for (int i = 0; i < C; ++i)
                q[o][i] = (double)Q[o * C + i];
        small_det_inv<C>(q, qi);
#pragma unroll
        for (int o = 0; o < C; ++o)
#pragma unroll
            for (int i = 0; i < C; ++i)
                if (tid == o * C + i)
                    sQinvT[tid] = (float)qi[i][o];
    }
    __syncthreads();
    for (int e = tid; e < E; e += 1024) {
        double total = swave[0][e];
#pragma unroll
        for (int v = 1; v < NW; ++v)
            total += swave[v][e];
        ssum[e] = (float)total;
    }
    __syncthreads();
    flow_finish_body(ssum, 1, w, s, b, Q, sQinvT, dLdw, dLds, dLdb, dLdQ, lw, C, H, W, k, tid, 1024);
}

// ---------------------------------------------------------------------------
// Fused forward, few channels, image in LDS: one wave per image brings y in with 16-byte accesses of
// consecutive lanes, solves in place (the single-wave systolic solve) and writes z = A x + d, four pixels
// of all channels per lane and trip.  x never reaches memory.
// ---------------------------------------------------------------------------
template <int C, int K>
__global__ __launch_bounds__(64) void k_flow_fwd_tile(const float *__restrict__ y, const float *__restrict__ w,
                                                     const float *__restrict__ mats, float *__restrict__ z, int H,
                                                     int W)
{
    extern __shared__ float smem[];
    const int n4 = C * H * W / 4, q4 = H * W / 4, lane = threadIdx.x;
    const float4 *src = reinterpret_cast<const float4 *>(y + (size_t)blockIdx.x * C * H * W);
    float4 *tile = reinterpret_cast<float4 *>(smem);
    for (int i = lane; i < n4; i += 8 * 64) {
        float4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            v[u] = src[i + 64 * u < n4 ? i + 64 * u : n4 - 1];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (i + 64 * u < n4)
                tile[i + 64 * u] = v[u];
    }
    float A[C][C], d[C];
#pragma unroll
    for (int o = 0; o < C; ++o) {
        d[o] = mats[flow_off_d(C) + o];
#pragma unroll
        for (int i = 0; i < C; ++i)
            A[o][i] = mats[o * C + i];
    }
    solve_wave_body<C, K, 0, false, false, true>(y, w, z, H, W, blockIdx.x, smem);
    f32x4 *dst = reinterpret_cast<f32x4 *>(z + (size_t)blockIdx.x * C * H * W);
    const f32x4 *t4 = reinterpret_cast<const f32x4 *>(smem);
    for (int q = lane; q < q4; q += 64) {
        f32x4 xin[C];
#pragma unroll
        for (int i = 0; i < C; ++i)
            xin[i] = t4[i * q4 + q];
#pragma unroll
        for (int o = 0; o < C; ++o) {
            f32x4 acc = f32x4{d[o], d[o], d[o], d[o]};
#pragma unroll
            for (int i = 0; i < C; ++i)
                acc += A[o][i] * xin[i];
            dst[o * q4 + q] = acc;
        }
    }
}

// ---------------------------------------------------------------------------
// Fused backward, few channels, image in LDS (four waves per image):
//   all waves   bring dL/dz and z in, four pixels of all channels per lane and trip, and leave three tiles
//               in LDS: g = A^T dL/dz (input of the transposed solve), x = A^-1 z + e with a zero halo (for the
//               weight gradient), and dL/dz itself (for M2, m1);
//   wave 0      transposed solve in place: g becomes v = dL/dy;
//   all waves   write v out, then form the image's sums as outer products on the matrix cores
//               (v_mfma_f32_4x4x1, 16 pixels per instruction): sum v[o] x[i][p - tap] for dL/dw and, with
//               dL/dz as the other operand, sum dL/dz[o] x[i][p] and sum dL/dz[o];
//               fixed-order reduction through LDS to one row [P | C*C | C] per image.
// ---------------------------------------------------------------------------
template <int C, int K>
__global__ __launch_bounds__(256) void k_flow_bwd_tile(const float *__restrict__ z, const float *__restrict__ w,
                                                      const float *__restrict__ gz, const float *__restrict__ mats,
                                                      float *__restrict__ v, float *__restrict__ part, int H, int W)
{
    extern __shared__ float smem[];
    constexpr int NCOL = C * K * K, NS = (NCOL + 3) / 4, P = C * NCOL;
    constexpr int NC2 = C + 1, NS2 = (NC2 + 3) / 4, P2 = C * NC2;       // second operand: x[i] of the pixel, and 1
    constexpr int NST = NS + NS2, PT = P + P2;
    const int XR = H + K - 1, XW = W + K - 1, HW = H * W;
    float *sv = smem;                                   // [C][H][W]   g, then v
    float *sg = sv + C * HW;                            // [C][H][W]   dL/dz
    float *sx = sg + C * HW;                            // [C][XR][XW] x, origin at (-(K-1), -(K-1))
    float *sred = smem;                                 // reuses the tiles after the products
    const int n = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int q4 = HW / 4;

    float A[C][C], Ai[C][C], ev[C];
#pragma unroll
    for (int o = 0; o < C; ++o) {
        ev[o] = mats[flow_off_e(C) + o];
#pragma unroll
        for (int i = 0; i < C; ++i) {
            A[o][i] = mats[o * C + i];
            Ai[o][i] = mats[flow_off_Ainv(C) + o * C + i];
        }
    }
    for (int idx = tid; idx < C * XR * XW; idx += 256) {       // halo (and everything else) to zero first
        const int cc = idx % XW, rr = (idx / XW) % XR;
        if (rr < K - 1 || cc < K - 1)
            sx[idx] = 0.0f;
    }
    {
        const f32x4 *g4 = reinterpret_cast<const f32x4 *>(gz + (size_t)n * C * HW);
        const f32x4 *z4 = reinterpret_cast<const f32x4 *>(z + (size_t)n * C * HW);
        f32x4 *sv4 = reinterpret_cast<f32x4 *>(sv), *sg4 = reinterpret_cast<f32x4 *>(sg);
        for (int q = tid; q < q4; q += 256) {
            f32x4 gq[C], zq[C];
#pragma unroll
            for (int c = 0; c < C; ++c) {
                gq[c] = g4[c * q4 + q];
                zq[c] = z4[c * q4 + q];
            }
            const int p = 4 * q, r = p / W, c0 = p - r * W;      // W is a multiple of 4: the four pixels share a row
#pragma unroll
            for (int i = 0; i < C; ++i) {
                f32x4 gi = f32x4{0.f, 0.f, 0.f, 0.f}, xi = f32x4{ev[i], ev[i], ev[i], ev[i]};
#pragma unroll
                for (int o = 0; o < C; ++o) {
                    gi += A[o][i] * gq[o];
                    xi += Ai[i][o] * zq[o];
                }
                sv4[i * q4 + q] = gi;
                sg4[i * q4 + q] = gq[i];
                float *xd = sx + (i * XR + r + K - 1) * XW + c0 + K - 1;
                xd[0] = xi[0];
                xd[1] = xi[1];
                xd[2] = xi[2];
                xd[3] = xi[3];
            }
        }
    }
    __syncthreads();
    if (wave == 0)
        solve_wave_body<C, K, 1, false, false, true>(gz, w, v, H, W, n, sv);
    __syncthreads();
    {
        float4 *v4 = reinterpret_cast<float4 *>(v + (size_t)n * C * HW);
        const float4 *sv4 = reinterpret_cast<const float4 *>(sv);
        for (int i = tid; i < C * q4; i += 256)
            v4[i] = sv4[i];
    }
    // lane = (block b, j): first operand row o = j (of v, or of dL/dz), second operand column 4s + j.
    // Rows o >= C and columns past the last one are padding: they read valid data and are never used.
    const int j = lane & 3, b = lane >> 2;
    const int aoff = (j < C) ? j * HW : 0;
    int boff[NST];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const int col = (4 * s + j < NCOL) ? 4 * s + j : 0;
        const int i = col / (K * K), a = (col / K) % K, bb = col % K;
        boff[s] = (i * XR + a) * XW + bb;
    }
    bool one[NS2];
#pragma unroll
    for (int s = 0; s < NS2; ++s) {
        const int col = 4 * s + j;
        one[s] = col == C;
        boff[NS + s] = ((col < C ? col : 0) * XR + (K - 1)) * XW + (K - 1);
    }
    f32x4 acc[NST];
#pragma unroll
    for (int s = 0; s < NST; ++s)
        acc[s] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int ngroups = (HW + 15) / 16;
    for (int q = wave; q < ngroups; q += 4) {
        const int p = q * 16 + b;
        const bool pv = p < HW;
        const int pr = pv ? p / W : 0, pc = pv ? p - pr * W : 0;
        const float avl = sv[aoff + pr * W + pc], agl = sg[aoff + pr * W + pc];
        const float av = pv ? avl : 0.0f, ag = pv ? agl : 0.0f;     // pixels past the end contribute nothing
        const float *bp = sx + pr * XW + pc;
#pragma unroll
        for (int s = 0; s < NS; ++s)
            acc[s] = __builtin_amdgcn_mfma_f32_4x4x1f32(av, bp[boff[s]], acc[s], 0, 0, 0);
#pragma unroll
        for (int s = 0; s < NS2; ++s) {
            const float xv = bp[boff[NS + s]];
            acc[NS + s] = __builtin_amdgcn_mfma_f32_4x4x1f32(ag, one[s] ? 1.0f : xv, acc[NS + s], 0, 0, 0);
        }
    }
    __syncthreads();        // tiles no longer needed: reuse them for the reduction
#pragma unroll
    for (int s = 0; s < NST; ++s)
#pragma unroll
        for (int o = 0; o < 4; ++o)
            sred[tid * (NST * 4) + s * 4 + o] = acc[s][o];
    __syncthreads();
    // fixed-order sum in two levels: the 16 blocks of each wave, then the four waves
    float *swave = sred + 256 * NST * 4;     // [4][PT]
    for (int idx = tid; idx < 4 * PT; idx += 256) {
        const int e = idx % PT, wv = idx / PT;
        int o, s, jj;
        if (e < P) {
            o = e / NCOL;
            const int col = e % NCOL;
            s = col >> 2;
            jj = col & 3;
        } else {
            o = (e - P) / NC2;
            const int col = (e - P) % NC2;
            s = NS + (col >> 2);
            jj = col & 3;
        }
        float sum = 0.0f;
#pragma unroll
        for (int bb = 0; bb < 16; ++bb)
            sum += sred[(wv * 64 + bb * 4 + jj) * (NST * 4) + s * 4 + o];
        swave[wv * PT + e] = sum;
    }
    __syncthreads();
    // row layout: [P] dL/dw sums, [C*C] M2[o][i], [C] m1[o]
    for (int e = tid; e < PT; e += 256) {
        const float val = ((swave[e] + swave[PT + e]) + swave[2 * PT + e]) + swave[3 * PT + e];
        int dst = e;
        if (e >= P) {
            const int o = (e - P) / NC2, col = (e - P) % NC2;
            dst = col < C ? P + o * C + col : P + C * C + o;
        }
        part[(size_t)n * PT + dst] = val;
    }
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
static bool flow_fused_ck(int C, int k) { return (C == 3 && (k == 3 || k == 5)) || ((C == 1 || C == 2 || C == 4) && k == 3); }

static size_t flow_bwd_tile_lds(int C, int H, int W, int k)
{
    const size_t tiles = 2 * (size_t)C * H * W + (size_t)C * (H + k - 1) * (W + k - 1);
    const size_t nst = (size_t)(C * k * k + 3) / 4 + (size_t)(C + 1 + 3) / 4;
    const size_t red = 256 * nst * 4 + 4 * ((size_t)C * C * k * k + (size_t)C * (C + 1));
    return sizeof(float) * (tiles > red ? tiles : red);
}

// The fused kernels take few-channel images of at most 64 rows whose tiles fit LDS, with rows of whole
// 16-byte pieces (the binding of the tensors' alignment is checked at launch)
// Fusing pays once the bytes matter: at a few images the separate passes ride on the four-wave solve kernels,
// which have the shorter dependent step (measured, forward + backward of a step: 16 x 3x32x32 61.7 us fused
// against 61.4 us separate, 32 x 3x64x64 k=5 172 against 130 us; 1024 x 3x32x32 97 against 152 us,
// 4096 x 3x32x32 303 against 495 us, 1024 x 3x64x64 342 against 591 us).
bool flow_fused_preferred(int B, int C, int H, int W) { return (size_t)B * C * H * W * sizeof(float) >= (4u << 20); }

bool flow_fused_supported(int C, int H, int W, int k)
{
    return flow_fused_ck(C, k) && wave_supported(C, H, k) && (W % 4) == 0 &&
           (size_t)C * H * W * sizeof(float) <= 64 * 1024 && flow_bwd_tile_lds(C, H, W, k) <= kMaxLdsBytes;
}

size_t flow_stat_rows(int B, int HW) { return (size_t)B * ((HW + kFlowStatPix - 1) / kFlowStatPix); }

int launch_flow_prep(const float *w, const float *s, const float *b, const float *Q, float *mats, float *logdet, int C,
                     int H, int W, int k, hipStream_t stream)
{
    const size_t lds = sizeof(double) * ((size_t)2 * C * C + 3 * C) + sizeof(int) * (size_t)C;
    if (C > 16) {
        if (!ensure_dynamic_lds(reinterpret_cast<const void *>(&k_flow_prep<true>), lds) || lds > kMaxLdsBytes)
            return INVCONV_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(k_flow_prep<true>, dim3(1), dim3(1024), lds, stream, w, s, b, Q, mats, logdet, C, H, W, k);
    } else {
        if (!ensure_dynamic_lds(reinterpret_cast<const void *>(&k_flow_prep<false>), lds) || lds > kMaxLdsBytes)
            return INVCONV_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(k_flow_prep<false>, dim3(1), dim3(256), lds, stream, w, s, b, Q, mats, logdet, C, H, W, k);
    }
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

int launch_flow_affine(bool transposed, const float *in, const float *M, const float *add, float *out, int B, int C,
                       int HW, hipStream_t stream)
{
    return transposed ? launch_affine<true>(in, M, add, out, B, C, HW, stream)
                      : launch_affine<false>(in, M, add, out, B, C, HW, stream);
}

int launch_flow_stats(const float *gz, const float *x, float *rows, int B, int C, int HW, hipStream_t stream)
{
    const int chunks = (HW + kFlowStatPix - 1) / kFlowStatPix;
    const size_t lds = sizeof(float) * 2 * (size_t)C * kFlowStatPix;
    if (!ensure_dynamic_lds(reinterpret_cast<const void *>(&k_flow_stats), lds) || lds > kMaxLdsBytes)
        return INVCONV_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(k_flow_stats, dim3((unsigned)(B * chunks)), dim3(256), lds, stream, gz, x, rows, C, HW, chunks);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

static size_t flow_bwd_maps_lds(int C)
{
    return sizeof(float) * (3 * (size_t)C * kFlowStatStride + 2 * (size_t)C * C + C);
}

bool flow_bwd_maps_supported(int C) { return flow_bwd_maps_lds(C) <= kMaxLdsBytes; }

// x, g and flow_stat_rows(B, HW) rows of [C*C | C] partial sums
int launch_flow_bwd_maps(const float *z, const float *gz, const float *mats, float *x, float *g, float *rows, int B,
                         int C, int HW, hipStream_t stream)
{
    const int chunks = (HW + kFlowStatPix - 1) / kFlowStatPix;
    const size_t lds = flow_bwd_maps_lds(C);
    if (!ensure_dynamic_lds(reinterpret_cast<const void *>(&k_flow_bwd_maps), lds) || lds > kMaxLdsBytes)
        return INVCONV_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(k_flow_bwd_maps, dim3((unsigned)(B * chunks)), dim3(256), lds, stream, z, gz, mats, x, g, rows,
                       C, HW, chunks);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

int launch_flow_plane_sum(const float *gz, float *out, int planes, int HW, hipStream_t stream)
{
    hipLaunchKernelGGL(k_flow_plane_sum, dim3((unsigned)planes), dim3(256), 0, stream, gz, out, HW);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

int launch_rows_sum(const float *rows, int nrows, int stride, int E, float *out, hipStream_t stream)
{
    if (nrows >= 512)
        hipLaunchKernelGGL(k_rows_sum<16>, dim3((E + 63) / 64), dim3(1024), 0, stream, rows, nrows, stride, E, out);
    else
        hipLaunchKernelGGL(k_rows_sum<4>, dim3((E + 63) / 64), dim3(256), 0, stream, rows, nrows, stride, E, out);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

int launch_flow_finish(const float *sums, int have_dw, const float *w, const float *s, const float *b, const float *Q,
                       const float *mats, float *dLdw, float *dLds, float *dLdb, float *dLdQ, float lw, int C, int H,
                       int W, int k, hipStream_t stream)
{
    hipLaunchKernelGGL(k_flow_finish, dim3(1), dim3(256), 0, stream, sums, have_dw, w, s, b, Q, mats, dLdw, dLds, dLdb,
                       dLdQ, lw, C, H, W, k);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

int launch_flow_finish_rows(const float *rows, int nrows, const float *w, const float *s, const float *b,
                            const float *Q, float *dLdw, float *dLds, float *dLdb, float *dLdQ, float lw, int C, int H,
                            int W, int k, hipStream_t stream)
{
    if (C < 1 || C > 4 || k != 3 || nrows < 1)
        return INVCONV_ERR_VARIANT;
    switch (C) {
    case 1: hipLaunchKernelGGL((k_flow_finish_rows<1>), dim3(1), dim3(1024), 0, stream, rows, nrows, w, s, b, Q, dLdw, dLds, dLdb, dLdQ, lw, H, W, k); break;
    case 2: hipLaunchKernelGGL((k_flow_finish_rows<2>), dim3(1), dim3(1024), 0, stream, rows, nrows, w, s, b, Q, dLdw, dLds, dLdb, dLdQ, lw, H, W, k); break;
    case 3: hipLaunchKernelGGL((k_flow_finish_rows<3>), dim3(1), dim3(1024), 0, stream, rows, nrows, w, s, b, Q, dLdw, dLds, dLdb, dLdQ, lw, H, W, k); break;
    default: hipLaunchKernelGGL((k_flow_finish_rows<4>), dim3(1), dim3(1024), 0, stream, rows, nrows, w, s, b, Q, dLdw, dLds, dLdb, dLdQ, lw, H, W, k); break;
    }
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

template <int C, int K>
static int launch_flow_fwd_tile_ck(const float *y, const float *w, const float *mats, float *z, int B, int H, int W,
                                   hipStream_t stream)
{
    const size_t lds = sizeof(float) * (size_t)C * H * W;
    if (!ensure_dynamic_lds(reinterpret_cast<const void *>(&k_flow_fwd_tile<C, K>), lds))
        return INVCONV_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((k_flow_fwd_tile<C, K>), dim3(B), dim3(64), lds, stream, y, w, mats, z, H, W);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

template <int C, int K>
static int launch_flow_bwd_tile_ck(const float *z, const float *w, const float *gz, const float *mats, float *v,
                                   float *part, int B, int H, int W, hipStream_t stream)
{
    const size_t lds = flow_bwd_tile_lds(C, H, W, K);
    if (!ensure_dynamic_lds(reinterpret_cast<const void *>(&k_flow_bwd_tile<C, K>), lds))
        return INVCONV_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((k_flow_bwd_tile<C, K>), dim3(B), dim3(256), lds, stream, z, w, gz, mats, v, part, H, W);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

int launch_flow_fwd_tile(const float *y, const float *w, const float *mats, float *z, int B, int C, int H, int W, int k,
                         hipStream_t stream)
{
    if (C == 3 && k == 3) return launch_flow_fwd_tile_ck<3, 3>(y, w, mats, z, B, H, W, stream);
    if (C == 3 && k == 5) return launch_flow_fwd_tile_ck<3, 5>(y, w, mats, z, B, H, W, stream);
    if (C == 1 && k == 3) return launch_flow_fwd_tile_ck<1, 3>(y, w, mats, z, B, H, W, stream);
    if (C == 2 && k == 3) return launch_flow_fwd_tile_ck<2, 3>(y, w, mats, z, B, H, W, stream);
    if (C == 4 && k == 3) return launch_flow_fwd_tile_ck<4, 3>(y, w, mats, z, B, H, W, stream);
    return INVCONV_ERR_VARIANT;
}

int launch_flow_bwd_tile(const float *z, const float *w, const float *gz, const float *mats, float *v, float *part,
                         int B, int C, int H, int W, int k, hipStream_t stream)
{
    if (C == 3 && k == 3) return launch_flow_bwd_tile_ck<3, 3>(z, w, gz, mats, v, part, B, H, W, stream);
    if (C == 3 && k == 5) return launch_flow_bwd_tile_ck<3, 5>(z, w, gz, mats, v, part, B, H, W, stream);
    if (C == 1 && k == 3) return launch_flow_bwd_tile_ck<1, 3>(z, w, gz, mats, v, part, B, H, W, stream);
    if (C == 2 && k == 3) return launch_flow_bwd_tile_ck<2, 3>(z, w, gz, mats, v, part, B, H, W, stream);
    if (C == 4 && k == 3) return launch_flow_bwd_tile_ck<4, 3>(z, w, gz, mats, v, part, B, H, W, stream);
    return INVCONV_ERR_VARIANT;
}

}  // namespace invconv
