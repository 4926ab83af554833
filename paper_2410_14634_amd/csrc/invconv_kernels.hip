// Shape-generic kernels of the inverse convolution: the anti-diagonal
// wavefront solve (both orientations), the weight-gradient correlation with
// its fixed-order reduction, the log-determinant, and the one-launch-per-
// anti-diagonal comparison variant.  gfx950 only.
#include <hip/hip_cooperative_groups.h>

#include <atomic>
#include <mutex>

#include "invconv_common.h"
#include "invconv_launch.h"

namespace invconv {

// ---------------------------------------------------------------------------
// Host-side caches of what the runtime says about a kernel
// ---------------------------------------------------------------------------
namespace {
struct LdsLimit { int dev; const void *fn; size_t bytes; };
struct Residency { int dev; const void *fn; int threads; size_t lds; int count; };
// fixed tables (no heap): a full table only means the runtime is asked again
constexpr int kCacheSlots = 512;
std::mutex g_cache_mutex;
LdsLimit g_lds_limits[kCacheSlots];
Residency g_residency[kCacheSlots];
int g_n_lds_limits = 0, g_n_residency = 0;
std::atomic<int> g_wait_budget{0};
}  // namespace

bool ensure_dynamic_lds(const void *fn, size_t bytes)
{
    if (bytes <= 48 * 1024)
        return true;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    std::lock_guard<std::mutex> lock(g_cache_mutex);
    for (int i = 0; i < g_n_lds_limits; ++i) {
        LdsLimit &e = g_lds_limits[i];
        if (e.dev == dev && e.fn == fn) {
            if (e.bytes >= bytes)
                return true;
            if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) {
                (void)hipGetLastError();
                return false;
            }
            e.bytes = bytes;
            return true;
        }
    }
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    if (g_n_lds_limits < kCacheSlots)
        g_lds_limits[g_n_lds_limits++] = LdsLimit{dev, fn, bytes};
    return true;
}

int resident_workgroups(const void *fn, int threads, size_t lds)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    std::lock_guard<std::mutex> lock(g_cache_mutex);
    for (int i = 0; i < g_n_residency; ++i) {
        const Residency &e = g_residency[i];
        if (e.dev == dev && e.fn == fn && e.threads == threads && e.lds == lds)
            return e.count;
    }
    int cus = 0, per_cu = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, threads, lds) != hipSuccess || cus < 1 ||
        per_cu < 1) {
        (void)hipGetLastError();
        return 0;
    }
    if (g_n_residency < kCacheSlots)
        g_residency[g_n_residency++] = Residency{dev, fn, threads, lds, cus * per_cu};
    return cus * per_cu;
}

int wait_budget(int standard)
{
    const int v = g_wait_budget.load(std::memory_order_relaxed);
    return v > 0 ? v : standard;
}

void set_wait_budget(int polls) { g_wait_budget.store(polls > 0 ? polls : 0, std::memory_order_relaxed); }

// ---------------------------------------------------------------------------
// Wavefront solve, one workgroup per image (Section 3.3: anti-diagonals in
// order, all pixels and channels of one anti-diagonal in parallel, one
// barrier per anti-diagonal).
//
// LDS holds the folded weights and a rolling window of the last 2(k-1)
// anti-diagonals of the solution plus the one being written, stored
// diagonal-major as win[d mod ND][row][channel] (row stride CP is odd so that
// lanes walking down a diagonal hit different banks).  Pixel (r,c) on diagonal
// d = r+c reads its neighbour (r-da, c-db) from diagonal d-da-db, row r-da.
// ---------------------------------------------------------------------------
// LEAN (many channels): no staging copy of the kernel in LDS, see fold_weights_lean.
template <int DIR, bool LEAN = false>
__global__ __launch_bounds__(kSolveBlock) void k_solve_block(const float *__restrict__ in,
                                                            const float *__restrict__ w,
                                                            float *__restrict__ out,
                                                            int C, int H, int W, int k)
{
    extern __shared__ float smem[];
    const int CP = C | 1;
    const int ND = 2 * (k - 1) + 1;
    float *sL = smem;
    float *sLinv = sL + C * C;
    float *sCf = sLinv + C * C;
    float *sW = sCf + k * k * C * C;
    float *win = LEAN ? sW : sW + k * k * C * C;

    const int n = blockIdx.x;
    const int tid = threadIdx.x;
    if (LEAN)
        fold_weights_lean<DIR>(w, C, k, sL, sLinv, sCf);
    else
        fold_weights<DIR>(w, C, k, sL, sLinv, sCf, sW);

    const int ndiag = H + W - 1;
    for (int d = 0; d < ndiag; ++d) {
        const int rlo = d - (W - 1) > 0 ? d - (W - 1) : 0;
        const int rhi = d < H - 1 ? d : H - 1;
        const int npx = rhi - rlo + 1;
        const int items = npx * C;
        const int slot_d = d % ND;
        for (int it = tid; it < items; it += kSolveBlock) {
            const int px = it % npx, o = it / npx;
            const int r = rlo + px, c = d - r;
            float acc = 0.0f;
            for (int j = 0; j <= o; ++j)
                acc += sLinv[o * C + j] * in[gidx<DIR>(n, j, r, c, C, H, W)];
            for (int da = 0; da < k && da <= r; ++da)
                for (int db = (da == 0) ? 1 : 0; db < k && db <= c; ++db) {
                    int slot = slot_d - (da + db);
                    if (slot < 0)
                        slot += ND;
                    const float *xw = win + (slot * H + (r - da)) * CP;
                    const float *cf = sCf + ((da * k + db) * C + o) * C;
                    for (int i = 0; i < C; ++i)
                        acc -= cf[i] * xw[i];
                }
            win[(slot_d * H + r) * CP + o] = acc;
            out[gidx<DIR>(n, o, r, c, C, H, W)] = acc;
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// Comparison variant: one launch per anti-diagonal.  One thread per
// (image, pixel of the diagonal); the thread solves its pixel's channels in
// order with the unfolded kernel, reading neighbours from `out` in global
// memory (written by earlier launches on the same stream).
// ---------------------------------------------------------------------------
template <int DIR>
__global__ __launch_bounds__(256) void k_solve_one_diagonal(const float *__restrict__ in,
                                                           const float *__restrict__ w,
                                                           float *out, int B, int C, int H, int W,
                                                           int k, int d)
{
    const int rlo = d - (W - 1) > 0 ? d - (W - 1) : 0;
    const int rhi = d < H - 1 ? d : H - 1;
    const int npx = rhi - rlo + 1;
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= B * npx)
        return;
    const int n = t / npx, r = rlo + t % npx, c = d - r;
    for (int o = 0; o < C; ++o) {
        float acc = in[gidx<DIR>(n, o, r, c, C, H, W)];
        for (int da = 0; da < k && da <= r; ++da)
            for (int db = (da == 0) ? 1 : 0; db < k && db <= c; ++db)
                for (int i = 0; i < C; ++i)
                    acc -= weff<DIR>(w, C, k, o, i, k - 1 - da, k - 1 - db) *
                           out[gidx<DIR>(n, i, r - da, c - db, C, H, W)];
        for (int i = 0; i < o; ++i)
            acc -= weff<DIR>(w, C, k, o, i, k - 1, k - 1) * out[gidx<DIR>(n, i, r, c, C, H, W)];
        out[gidx<DIR>(n, o, r, c, C, H, W)] = acc / weff<DIR>(w, C, k, o, o, k - 1, k - 1);
    }
}

// ---------------------------------------------------------------------------
// Last resort of the default path, for shapes that no on-chip kernel holds (more than 48 channels, or a
// window that outgrows LDS): one launch per anti-diagonal as above, but one WAVE per (image, pixel).  The
// C k k values the pixel's channels all read - its neighbours' x, and its own channels as they become known -
// sit in LDS, term t = (i k + a) k + b at sval[t]; for output channel o the lanes share the dot product with
// row o of the kernel (contiguous in t for the forward orientation), a butterfly adds the 64 partial sums,
// and the new x_o takes its place among the values before channel o + 1 starts (Eq. 1 solved for x, channel
// by channel).  Two to three orders of magnitude faster than a thread per pixel at 64 channels.
// ---------------------------------------------------------------------------
// MAXJ: terms of a kernel row per lane that the registers hold (16, 40 or 64: rows of up to 1024, 2560 or 4096
// entries); longer rows are read where they are used.
template <int DIR, int MAXJ>
__global__ __launch_bounds__(256) void k_solve_diag_wave(const float *__restrict__ in, const float *__restrict__ w,
                                                        float *out, int B, int C, int H, int W, int k, int d)
{
    extern __shared__ float sval_all[];
    const int lane = threadIdx.x & 63, wv_in_block = threadIdx.x >> 6;
    const int rlo = d - (W - 1) > 0 ? d - (W - 1) : 0;
    const int rhi = d < H - 1 ? d : H - 1;
    const int npx = rhi - rlo + 1;
    const long long item = (long long)blockIdx.x * 4 + wv_in_block;
    if (item >= (long long)B * npx)
        return;                                 // (no barrier in this kernel)
    const int n = (int)(item / npx), r = rlo + (int)(item % npx), c = d - r;
    const int T = C * k * k;
    float *sval = sval_all + (size_t)wv_in_block * T;
    for (int t = lane; t < T; t += 64) {
        const int b = t % k, a = (t / k) % k, i = t / (k * k);
        const int da = k - 1 - a, db = k - 1 - b;
        float v = 0.0f;                         // the pixel's own channels: not known yet
        if ((da || db) && da <= r && db <= c)
            v = out[gidx<DIR>(n, i, r - da, c - db, C, H, W)];
        sval[t] = v;
    }
    __builtin_amdgcn_wave_barrier();
    // Row o + 1 of the kernel (this lane's terms), its diagonal entry and y_{o+1} are fetched while channel o is
    // being solved: the chain over the channels then waits for LDS and the butterfly only, not for memory.
    const int nj = (T + 63) / 64;
    const bool pre = nj <= MAXJ;
    // where this lane's terms sit in a row of the kernel (no division in the loop over the channels): entry
    // (o, t) is at toff + o T in the forward orientation; mirrored, w'[o][i][a][b] = w[C-1-i][C-1-o][a][b] is at
    // toff + (C-1-o) k k.  curi: the term's channel if it is a current-pixel tap (masked for i > o), else -1.
    int toff[MAXJ], curi[MAXJ];
    const int kk = k * k;
#pragma unroll
    for (int j = 0; j < MAXJ; ++j) {
        const int t = lane + 64 * j;
        const int tc = t < T ? t : T - 1;
        const int ab = tc % kk, i = tc / kk;
        toff[j] = DIR ? (C - 1 - i) * C * kk + ab : tc;
        curi[j] = (t < T && ab == kk - 1) ? i : (t < T ? -1 : C);       // (terms past the row: always masked)
    }
    float wrow[MAXJ], wdiag = 1.0f, yo = 0.0f;
    auto fetch = [&](int o) {
        const int oc = o < C ? o : C - 1;
        const int obase = DIR ? (C - 1 - oc) * kk : oc * T;
#pragma unroll
        for (int j = 0; j < MAXJ; ++j) {
            const float v = j < nj ? w[obase + toff[j]] : 0.0f;
            wrow[j] = curi[j] > oc ? 0.0f : v;
        }
        const int od = DIR ? C - 1 - oc : oc;
        wdiag = w[(od * C + od) * kk + kk - 1];
        yo = in[gidx<DIR>(n, oc, r, c, C, H, W)];
    };
    if (pre)
        fetch(0);
    for (int o = 0; o < C; ++o) {
        float part = 0.0f, diag, yv;
        if (pre) {
#pragma unroll
            for (int j = 0; j < MAXJ; ++j)
                if (j < nj)
                    part += wrow[j] * sval[lane + 64 * j < T ? lane + 64 * j : 0];
            diag = wdiag;
            yv = yo;
            fetch(o + 1);
        } else {
            for (int t = lane; t < T; t += 64) {
                const int b = t % k, a = (t / k) % k, i = t / (k * k);
                part += weff<DIR>(w, C, k, o, i, a, b) * sval[t];
            }
            diag = weff<DIR>(w, C, k, o, o, k - 1, k - 1);
            yv = in[gidx<DIR>(n, o, r, c, C, H, W)];
        }
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1)
            part += __shfl_xor(part, m, 64);
        const float xo = (yv - part) / diag;
        if (lane == 0) {
            out[gidx<DIR>(n, o, r, c, C, H, W)] = xo;
            sval[(o * k + (k - 1)) * k + (k - 1)] = xo;     // the current-pixel tap of channel o
        }
        __builtin_amdgcn_wave_barrier();        // (LDS operations of a wave complete in order)
    }
}

// ---------------------------------------------------------------------------
// Comparison variant: ONE cooperative launch of a persistent grid that walks
// the anti-diagonals itself and separates them with a device-wide barrier
// (cooperative-groups grid sync).  Same per-pixel work as the launch-per-
// diagonal variant; every (image, pixel) of a diagonal is one work item and
// the grid strides over them, so an image may be spread over many compute units.
// ---------------------------------------------------------------------------
template <int DIR>
__global__ __launch_bounds__(256) void k_solve_persistent(const float *__restrict__ in,
                                                         const float *__restrict__ w, float *out, int B,
                                                         int C, int H, int W, int k)
{
    namespace cg = cooperative_groups;
    cg::grid_group grid = cg::this_grid();
    const int ndiag = H + W - 1;
    const int nthreads = gridDim.x * blockDim.x;
    const int t0 = blockIdx.x * blockDim.x + threadIdx.x;
    for (int d = 0; d < ndiag; ++d) {
        const int rlo = d - (W - 1) > 0 ? d - (W - 1) : 0;
        const int rhi = d < H - 1 ? d : H - 1;
        const int npx = rhi - rlo + 1;
        for (int t = t0; t < B * npx; t += nthreads) {
            const int n = t / npx, r = rlo + t % npx, c = d - r;
            for (int o = 0; o < C; ++o) {
                float acc = in[gidx<DIR>(n, o, r, c, C, H, W)];
                for (int da = 0; da < k && da <= r; ++da)
                    for (int db = (da == 0) ? 1 : 0; db < k && db <= c; ++db)
                        for (int i = 0; i < C; ++i)
                            acc -= weff<DIR>(w, C, k, o, i, k - 1 - da, k - 1 - db) *
                                   out[gidx<DIR>(n, i, r - da, c - db, C, H, W)];
                for (int i = 0; i < o; ++i)
                    acc -= weff<DIR>(w, C, k, o, i, k - 1, k - 1) * out[gidx<DIR>(n, i, r, c, C, H, W)];
                out[gidx<DIR>(n, o, r, c, C, H, W)] = acc / weff<DIR>(w, C, k, o, o, k - 1, k - 1);
            }
        }
        grid.sync();    // every thread of the grid reaches this once per diagonal
    }
}

// ---------------------------------------------------------------------------
// Step-synchronisation probes: the cost of one dependent step under each of the
// three ways of ordering anti-diagonals, with no arithmetic in between.
// ---------------------------------------------------------------------------
__global__ void k_probe_empty(int *sink)
{
    if (sink && threadIdx.x == 1000000)
        sink[0] = 0;
}

__global__ __launch_bounds__(256) void k_probe_grid_sync(int steps, int *sink)
{
    namespace cg = cooperative_groups;
    cg::grid_group grid = cg::this_grid();
    for (int s = 0; s < steps; ++s)
        grid.sync();
    if (sink && threadIdx.x == 1000000)
        sink[0] = 0;
}

__global__ __launch_bounds__(256) void k_probe_block_sync(int steps, int *sink)
{
    __shared__ float buf[256];
    float v = threadIdx.x;
    for (int s = 0; s < steps; ++s) {
        buf[threadIdx.x] = v;
        __syncthreads();
        v += buf[(threadIdx.x + 64) & 255];
        __syncthreads();
    }
    if (sink && v == -1.0f)
        sink[0] = 0;
}

int launch_probe(int mode, int steps, int blocks, hipStream_t stream)
{
    int *sink = nullptr;
    if (mode == 0) {
        for (int s = 0; s < steps; ++s)
            hipLaunchKernelGGL(k_probe_empty, dim3(blocks), dim3(256), 0, stream, sink);
    } else if (mode == 1) {
        void *args[] = {(void *)&steps, (void *)&sink};
        if (hipLaunchCooperativeKernel(reinterpret_cast<void *>(k_probe_grid_sync), dim3(blocks), dim3(256), args, 0,
                                       stream) != hipSuccess) {
            (void)hipGetLastError();
            return INVCONV_ERR_LAUNCH;
        }
    } else {
        hipLaunchKernelGGL(k_probe_block_sync, dim3(blocks), dim3(256), 0, stream, steps, sink);
    }
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

// ---------------------------------------------------------------------------
// Weight gradient, pass 1 (Eq. 4 with Theorem 2):
//   dw[o][i][a][b] = - sum_{n,r,c} v[n][o][r][c] * x[n][i][r-(k-1)+a][c-(k-1)+b].
// One workgroup per (image, chunk of RT rows x CW columns) stages v and x (with
// a halo of k-1 rows/columns on the top/left, zero outside the image) in LDS
// and writes the un-negated
// partial sums of all P = C*C*k*k entries to part[workgroup][P].  When P is
// smaller than the block, G = block/P thread groups split the pixels and are
// combined in a fixed order through LDS.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kDwBlock) void k_dw_partial(const float *__restrict__ x,
                                                        const float *__restrict__ v,
                                                        float *__restrict__ part,
                                                        int C, int H, int W, int k, int RT, int nchunks, int CW, int ncol)
{
    extern __shared__ float smem[];
    const int per_image = nchunks * ncol;
    const int n = blockIdx.x / per_image, chunk = (blockIdx.x % per_image) / ncol, cchunk = blockIdx.x % ncol;
    const int r0 = chunk * RT, c0 = cchunk * CW;
    const int rows = (H - r0 < RT) ? H - r0 : RT;
    const int cols = (W - c0 < CW) ? W - c0 : CW;
    const int XR = RT + k - 1, XW = CW + k - 1;
    const int P = C * C * k * k;
    const int G = (P < kDwBlock) ? kDwBlock / P : 1;
    float *sv = smem;                 // [C][RT][CW]
    float *sx = sv + C * RT * CW;     // [C][XR][XW], origin at (r0-(k-1), c0-(k-1))
    float *sred = sx + C * XR * XW;   // [G][P] when G > 1
    const int tid = threadIdx.x;

    for (int idx = tid; idx < C * rows * cols; idx += kDwBlock) {
        const int c = idx % cols, r = (idx / cols) % rows, ch = idx / (cols * rows);
        sv[(ch * RT + r) * CW + c] = v[(((size_t)n * C + ch) * H + r0 + r) * W + c0 + c];
    }
    const int xrows = rows + k - 1, xcols = cols + k - 1;
    for (int idx = tid; idx < C * xrows * xcols; idx += kDwBlock) {
        const int cc = idx % xcols, rr = (idx / xcols) % xrows, ch = idx / (xcols * xrows);
        const int gr = r0 - (k - 1) + rr, gc = c0 - (k - 1) + cc;
        sx[(ch * XR + rr) * XW + cc] =
            (gr >= 0 && gc >= 0) ? x[(((size_t)n * C + ch) * H + gr) * W + gc] : 0.0f;
    }
    __syncthreads();

    const int lanesE = (G > 1) ? P : kDwBlock;
    const int s = tid / lanesE, e0 = tid % lanesE;
    const int npix = rows * cols;
    if (s < G) {
        for (int e = e0; e < P; e += lanesE) {
            const int b = e % k, a = (e / k) % k, i = (e / (k * k)) % C, o = e / (k * k * C);
            const float *pv = sv + o * RT * CW;
            const float *px = sx + (i * XR + a) * XW + b;
            float acc = 0.0f;
            for (int p = s; p < npix; p += G) {
                const int r = p / cols, c = p - r * cols;
                acc += pv[r * CW + c] * px[r * XW + c];
            }
            if (G > 1)
                sred[s * P + e] = acc;
            else
                part[(size_t)blockIdx.x * P + e] = acc;
        }
    }
    if (G > 1) {
        __syncthreads();
        if (tid < P) {
            float acc = 0.0f;
            for (int g = 0; g < G; ++g)
                acc += sred[g * P + tid];
            part[(size_t)blockIdx.x * P + tid] = acc;
        }
    }
}

// Pass 2: a workgroup takes 64 consecutive kernel entries (lanes, so that every
// row of `part` is read in 256-byte pieces); its four waves add the rows
// p = wave, wave+4, ... in index order (double accumulator) and are then
// combined in wave order.  The result is negated and masked entries are written
// as 0.  No atomics anywhere, so dw is bitwise reproducible from run to run.
// blockIdx.y selects the layer when several layers are reduced by one launch
// (layer l's rows start at part + l*nparts*P, its result goes to out.p[l]).
// Rows may hold one Cv x C block of a larger result (entries for output channels o0 .. and input channels i0 .. of a
// Ctot-channel kernel gradient); the launches here pass the whole result, results formed in blocks take
// k_dw_reduce_blocks below.
template <int NW>
__global__ __launch_bounds__(64 * NW) void k_dw_reduce(const float *__restrict__ part_all, int nparts, PtrList out,
                                                      int C, int k, float sign, int Cv, int o0, int i0, int Ctot)
{
    // NW = 4 waves, or 16 for many rows (the launch decides from nparts alone, so the order of the additions
    // is a function of the shape): wave v adds rows v, v + NW, ... in order, then the waves are added in order
    __shared__ double swave[NW][64];
    const int P = Cv * C * k * k;
    const float *__restrict__ part = part_all + (size_t)blockIdx.y * nparts * P;
    float *__restrict__ dw = out.p[blockIdx.y];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int e = blockIdx.x * 64 + lane;
    double acc = 0.0;
    if (e < P) {
        int p = wave;
        for (; p + 7 * NW < nparts; p += 8 * NW) {
            float a[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                a[u] = part[(size_t)(p + NW * u) * P + e];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                acc += (double)a[u];
        }
        // the last rows: loaded together as well (addresses clamped, rows past the end count as zero), so that
        // few rows cost one memory latency, not one per row
        if (p < nparts) {
            float a[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int r = p + NW * u;
                a[u] = part[(size_t)(r < nparts ? r : nparts - 1) * P + e];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                acc += p + NW * u < nparts ? (double)a[u] : 0.0;
        }
    }
    swave[wave][lane] = acc;
    __syncthreads();
    if (wave == 0 && e < P) {
        double total = swave[0][lane];
#pragma unroll
        for (int v = 1; v < NW; ++v)
            total += swave[v][lane];
        const int b = e % k, a = (e / k) % k, i = i0 + (e / (k * k)) % C, o = o0 + e / (k * k * C);
        const bool is_masked = (a == k - 1 && b == k - 1 && i > o);
        dw[((o * Ctot + i) * k + a) * k + b] = is_masked ? 0.0f : (float)(sign < 0.0f ? -total : total);
    }
}

// The same second pass for the blocks of a result with more than 16 channels, all in one launch: blockIdx.y
// selects the block (its channel counts and its place in the result come from `blocks`).
template <int NW>
__global__ __launch_bounds__(64 * NW) void k_dw_reduce_blocks(const float *__restrict__ part_all, int nparts,
                                                             float *__restrict__ dw, DwBlocks blocks, int Ctot, int k,
                                                             int pstride, float sign, int masked)
{
    __shared__ double swave[NW][64];
    const int y = blockIdx.y;
    const int Cv = blocks.cv[y], C = blocks.cx[y], o0 = blocks.o0[y], i0 = blocks.i0[y];
    const int P = Cv * C * k * k;
    const float *__restrict__ part = part_all + (size_t)y * nparts * pstride;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int e = blockIdx.x * 64 + lane;
    double acc = 0.0;
    if (e < P) {
        // rows wave, wave + NW, ... in index order, eight loads in flight (addresses clamped, rows past the end
        // count as zero)
        for (int p = wave; p < nparts; p += 8 * NW) {
            float a[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int r = p + NW * u;
                a[u] = part[(size_t)(r < nparts ? r : nparts - 1) * pstride + e];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                acc += p + NW * u < nparts ? (double)a[u] : 0.0;
        }
    }
    swave[wave][lane] = acc;
    __syncthreads();
    if (wave == 0 && e < P) {
        double total = swave[0][lane];
#pragma unroll
        for (int v = 1; v < NW; ++v)
            total += swave[v][lane];
        const int b = e % k, a = (e / k) % k, i = i0 + (e / (k * k)) % C, o = o0 + e / (k * k * C);
        const bool is_masked = masked && (a == k - 1 && b == k - 1 && i > o);
        dw[((o * Ctot + i) * k + a) * k + b] = is_masked ? 0.0f : (float)(sign < 0.0f ? -total : total);
    }
}

// log|det dx/dy| for one image (Section 4): -H*W*sum_c log|w[c][c][k-1][k-1]|.
// One wave; lane l takes channels l, l+64, ...; fixed butterfly across lanes.
// blockIdx.x selects the layer: kernel ws.p[l], result out[l].
__global__ __launch_bounds__(64) void k_logdet(ConstPtrList ws, int C, int H, int W, int k,
                                              float *__restrict__ out_all)
{
    const float *__restrict__ w = ws.p[blockIdx.x];
    float *__restrict__ out = out_all + blockIdx.x;
    double s = 0.0;
    for (int c = threadIdx.x; c < C; c += 64)
        s += log(fabs((double)w[((c * C + c) * k + (k - 1)) * k + (k - 1)]));
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1)
        s += __shfl_xor(s, m, 64);
    if (threadIdx.x == 0)
        out[0] = (float)(-(double)H * (double)W * s);
}

// ---------------------------------------------------------------------------
// Host-side launchers
// ---------------------------------------------------------------------------
static size_t solve_block_lds_bytes_form(int C, int H, int k, bool lean)
{
    const size_t CP = (size_t)(C | 1), ND = 2 * (size_t)(k - 1) + 1;
    return sizeof(float) * (2 * (size_t)C * C + (lean ? 1 : 2) * (size_t)k * k * C * C + ND * H * CP);
}

// What the launch will take: the form with the staging buffer while it fits, the lean one beyond
size_t solve_block_lds_bytes(int C, int H, int k)
{
    const size_t full = solve_block_lds_bytes_form(C, H, k, false);
    return full <= kMaxLdsBytes ? full : solve_block_lds_bytes_form(C, H, k, true);
}

template <int DIR>
static int launch_solve_block_dir(const float *in, const float *w, float *out, int B, int C, int H, int W,
                                  int k, hipStream_t stream)
{
    const size_t lds = solve_block_lds_bytes(C, H, k);
    if (lds > kMaxLdsBytes)
        return INVCONV_ERR_UNSUPPORTED;
    const bool lean = solve_block_lds_bytes_form(C, H, k, false) > kMaxLdsBytes;
    const void *fn = lean ? reinterpret_cast<const void *>(&k_solve_block<DIR, true>)
                          : reinterpret_cast<const void *>(&k_solve_block<DIR, false>);
    if (!ensure_dynamic_lds(fn, lds))
        return INVCONV_ERR_UNSUPPORTED;
    if (lean)
        hipLaunchKernelGGL((k_solve_block<DIR, true>), dim3(B), dim3(kSolveBlock), lds, stream, in, w, out, C, H, W, k);
    else
        hipLaunchKernelGGL((k_solve_block<DIR, false>), dim3(B), dim3(kSolveBlock), lds, stream, in, w, out, C, H, W,
                           k);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

int launch_solve_block(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W,
                       int k, hipStream_t stream)
{
    return dir ? launch_solve_block_dir<1>(in, w, out, B, C, H, W, k, stream)
               : launch_solve_block_dir<0>(in, w, out, B, C, H, W, k, stream);
}

int launch_solve_diag(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W,
                      int k, hipStream_t stream)
{
    const int ndiag = H + W - 1;
    for (int d = 0; d < ndiag; ++d) {
        const int rlo = d - (W - 1) > 0 ? d - (W - 1) : 0;
        const int rhi = d < H - 1 ? d : H - 1;
        const long long items = (long long)B * (rhi - rlo + 1);
        const int grid = (int)((items + 255) / 256);
        if (dir)
            hipLaunchKernelGGL(k_solve_one_diagonal<1>, dim3(grid), dim3(256), 0, stream, in, w, out, B, C,
                               H, W, k, d);
        else
            hipLaunchKernelGGL(k_solve_one_diagonal<0>, dim3(grid), dim3(256), 0, stream, in, w, out, B, C,
                               H, W, k, d);
        if (hipGetLastError() != hipSuccess)
            return INVCONV_ERR_LAUNCH;
    }
    return INVCONV_OK;
}

template <int DIR>
static int launch_persistent_dir(const float *in, const float *w, float *out, int B, int C, int H, int W, int k,
                                 hipStream_t stream)
{
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_solve_persistent<DIR>, 256, 0) != hipSuccess ||
        cus < 1 || per_cu < 1) {
        (void)hipGetLastError();
        return INVCONV_ERR_LAUNCH;
    }
    const int longest = H < W ? H : W;
    long long want = ((long long)B * longest + 255) / 256;      // enough threads for the longest diagonal
    const long long cap = (long long)cus * per_cu;              // what can be resident at once
    if (want > cap) want = cap;
    if (want < 1) want = 1;
    void *args[] = {(void *)&in, (void *)&w, (void *)&out, (void *)&B, (void *)&C, (void *)&H, (void *)&W, (void *)&k};
    if (hipLaunchCooperativeKernel(reinterpret_cast<void *>(k_solve_persistent<DIR>), dim3((unsigned)want), dim3(256),
                                   args, 0, stream) != hipSuccess) {
        (void)hipGetLastError();
        return INVCONV_ERR_LAUNCH;
    }
    return INVCONV_OK;
}

// one launch per anti-diagonal, a wave per pixel (see k_solve_diag_wave); refuses kernels of more than 8192
// entries per output channel (four waves' values have to fit 128 KB of LDS)
template <int DIR, int MAXJ>
static int launch_diag_wave_dj(const float *in, const float *w, float *out, int B, int C, int H, int W, int k,
                               hipStream_t stream)
{
    const size_t lds = 4 * (size_t)C * k * k * sizeof(float);
    if (!ensure_dynamic_lds(reinterpret_cast<const void *>(&k_solve_diag_wave<DIR, MAXJ>), lds))
        return INVCONV_ERR_UNSUPPORTED;
    const int ndiag = H + W - 1;
    for (int d = 0; d < ndiag; ++d) {
        const int rlo = d - (W - 1) > 0 ? d - (W - 1) : 0;
        const int rhi = d < H - 1 ? d : H - 1;
        const long long items = (long long)B * (rhi - rlo + 1);
        const unsigned grid = (unsigned)((items + 3) / 4);
        hipLaunchKernelGGL((k_solve_diag_wave<DIR, MAXJ>), dim3(grid), dim3(256), lds, stream, in, w, out, B, C, H, W, k,
                           d);
        if (hipGetLastError() != hipSuccess)
            return INVCONV_ERR_LAUNCH;
    }
    return INVCONV_OK;
}

int launch_solve_diag_wave(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W, int k,
                           hipStream_t stream)
{
    const size_t T = (size_t)C * k * k;
    if (T > 8192)
        return INVCONV_ERR_UNSUPPORTED;
    if (T <= 1024)
        return dir ? launch_diag_wave_dj<1, 16>(in, w, out, B, C, H, W, k, stream)
                   : launch_diag_wave_dj<0, 16>(in, w, out, B, C, H, W, k, stream);
    if (T <= 2560)
        return dir ? launch_diag_wave_dj<1, 40>(in, w, out, B, C, H, W, k, stream)
                   : launch_diag_wave_dj<0, 40>(in, w, out, B, C, H, W, k, stream);
    return dir ? launch_diag_wave_dj<1, 64>(in, w, out, B, C, H, W, k, stream)
               : launch_diag_wave_dj<0, 64>(in, w, out, B, C, H, W, k, stream);
}

int launch_solve_persistent(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W,
                            int k, hipStream_t stream)
{
    return dir ? launch_persistent_dir<1>(in, w, out, B, C, H, W, k, stream)
               : launch_persistent_dir<0>(in, w, out, B, C, H, W, k, stream);
}

DwPlan plan_dw(int B, int C, int H, int W, int k)
{
    DwPlan p{};
    const size_t P = (size_t)C * C * k * k;
    const size_t G = P < (size_t)kDwBlock ? kDwBlock / P : 1;
    const size_t red = G > 1 ? G * P : 0;
    // largest row chunk whose tiles fit the LDS budget; an image too wide for one row is also cut into
    // column chunks
    auto lds_for = [&](int rt, int cw) {
        return sizeof(float) * ((size_t)C * rt * cw + (size_t)C * (rt + k - 1) * (cw + k - 1) + red);
    };
    int cw = W;
    while (cw > 1 && lds_for(1, cw) > kDwLdsBudget)
        cw = (cw + 1) / 2;
    if (lds_for(1, cw) > kDwLdsBudget)
        return p;   // rt == 0: unsupported
    int want = (int)((1024 + B - 1) / B);          // aim for about a thousand workgroups
    if (want < 1) want = 1;
    int rt = (H + want - 1) / want;
    if (rt < 1) rt = 1;
    while (rt > 1 && lds_for(rt, cw) > kDwLdsBudget)
        --rt;
    p.rt = rt;
    p.nchunks = (H + rt - 1) / rt;
    p.cw = cw;
    p.ncol = (W + cw - 1) / cw;
    p.nparts = (size_t)B * p.nchunks * p.ncol;
    p.lds = lds_for(rt, cw);
    p.bytes = ((p.nparts * P * sizeof(float)) + 255) / 256 * 256;
    return p;
}

// The plan invconv_bwd uses: matrix-core pass 1 when the shape allows it, the generic one otherwise.
// `bytes` also covers the one-row-per-image partials of the fused backward kernel.
DwPlan plan_dw_any(int B, int C, int H, int W, int k)
{
    DwPlan p = dw_mfma_supported(C, k) ? plan_dw_mfma(B, C, H, W, k) : DwPlan{};
    if (!p.rt)
        p = plan_dw(B, C, H, W, k);
    if (p.rt) {
        const size_t P = (size_t)C * C * k * k;
        const size_t per_image = (((size_t)B * P * sizeof(float)) + 255) / 256 * 256;
        if (p.bytes < per_image)
            p.bytes = per_image;
    }
    return p;
}

int launch_dw(const float *x, const float *v, float *dw, float *part, const DwPlan &p, int B, int C, int H,
              int W, int k, hipStream_t stream, float sign)
{
    hipLaunchKernelGGL(k_dw_partial, dim3((unsigned)p.nparts), dim3(kDwBlock), p.lds, stream, x, v, part, C, H,
                       W, k, p.rt, p.nchunks, p.cw, p.ncol);
    if (hipGetLastError() != hipSuccess)
        return INVCONV_ERR_LAUNCH;
    return launch_dw_reduce(part, (int)p.nparts, dw, C, k, stream, sign);
}

int launch_dw_reduce(const float *part, int nparts, float *dw, int C, int k, hipStream_t stream, float sign)
{
    return launch_dw_reduce_layers(part, nparts, &dw, 1, C, k, stream, sign);
}

// Second pass for `layers` layers in one launch (rows of layer l start at part + l*nparts*P).
int launch_dw_reduce_layers(const float *part, int nparts, float *const *dw, int layers, int C, int k,
                            hipStream_t stream, float sign)
{
    if (layers < 1 || layers > kChainMaxLayers)
        return INVCONV_ERR_SHAPE;
    const int P = C * C * k * k;
    PtrList out{};
    for (int l = 0; l < layers; ++l)
        out.p[l] = dw[l];
    if (nparts >= 512)
        hipLaunchKernelGGL(k_dw_reduce<16>, dim3((P + 63) / 64, layers), dim3(1024), 0, stream, part, nparts, out, C, k,
                           sign, C, 0, 0, C);
    else
        hipLaunchKernelGGL(k_dw_reduce<4>, dim3((P + 63) / 64, layers), dim3(256), 0, stream, part, nparts, out, C, k,
                           sign, C, 0, 0, C);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

int launch_dw_reduce_blocks(const float *part, int nparts, float *dw, const DwBlocks &blocks, int Ctot, int k,
                            int pstride, hipStream_t stream, float sign, bool masked)
{
    if (blocks.n < 1 || blocks.n > kChainMaxLayers)
        return INVCONV_ERR_SHAPE;
    const dim3 grid((pstride + 63) / 64, blocks.n);
    if (nparts >= 512)
        hipLaunchKernelGGL(k_dw_reduce_blocks<16>, grid, dim3(1024), 0, stream, part, nparts, dw, blocks, Ctot, k, pstride,
                           sign, masked ? 1 : 0);
    else
        hipLaunchKernelGGL(k_dw_reduce_blocks<4>, grid, dim3(256), 0, stream, part, nparts, dw, blocks, Ctot, k, pstride,
                           sign, masked ? 1 : 0);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

int launch_logdet(const float *w, int C, int H, int W, int k, float *out, hipStream_t stream)
{
    return launch_logdet_layers(&w, 1, C, H, W, k, out, stream);
}

int launch_logdet_layers(const float *const *w, int layers, int C, int H, int W, int k, float *out,
                         hipStream_t stream)
{
    if (layers < 1 || layers > kChainMaxLayers)
        return INVCONV_ERR_SHAPE;
    ConstPtrList ws{};
    for (int l = 0; l < layers; ++l)
        ws.p[l] = w[l];
    hipLaunchKernelGGL(k_logdet, dim3(layers), dim3(64), 0, stream, ws, C, H, W, k, out);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

}  // namespace invconv
