// The masked causal convolution itself, y = conv_w(x) (Eq. 1; the sampling
// direction of Section 4.3, which only needs plain convolutions).  Every output
// pixel is independent, so this is a streaming kernel: the images are cut into
// tiles of 16 rows; a workgroup walks a contiguous run of tiles, stages each
// tile of x (with a halo of k-1 rows above and columns to the left, zero
// outside the image) in LDS and forms all C output channels on the matrix
// cores.  gfx950 only.
//
//   C <= 4   v_mfma_f32_4x4x1: lane = pixel, the four result registers are the
//            output channels, one instruction per (input channel, tap);
//   else     v_mfma_f32_16x16x4: M = 16 pixels, N = 16 output channels, K = 4 of
//            the C*k*k (input channel, tap) pairs per instruction.
#include "invconv_common.h"
#include "invconv_launch.h"

namespace invconv {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kConvRows = 16;                   // tile height
constexpr int kConvLoadBatch = 8;               // loads in flight per thread while a tile is staged
constexpr size_t kConvLdsBudget = 72 * 1024;    // tile + tables; two workgroups per CU at the limit
constexpr int kConvMaxGrid = 1024;              // workgroups of a launch (four per CU)
constexpr int kConvMaxGridDw = 2048;            // ... of the launch that only forms weight-gradient sums (small tiles)

// n / d for n * d < 2^32 with m = magic(d): one multiply instead of a division sequence.
__device__ __forceinline__ unsigned magic(unsigned d) { return 0xFFFFFFFFu / d + 1u; }
__device__ __forceinline__ unsigned fastdiv(unsigned n, unsigned d, unsigned m) { return d == 1u ? n : __umulhi(n, m); }

// Workgroup ids are dealt round-robin to the 8 XCDs, each with an L2 of its own.  Tiles are numbered
// column-first, then row, then image, so neighbours in that order share halo rows and columns.
// Every XCD owns one contiguous eighth of the tiles and its workgroups sweep that range side by
// side (workgroup lw of n takes tiles first + lw, first + lw + n, ...): tiles in flight at the same
// time on an XCD are neighbours, so a halo is read from HBM once and found in that XCD's L2 after.
__device__ __forceinline__ void tile_sweep(unsigned ntiles, unsigned &first, unsigned &last, unsigned &stride)
{
    const unsigned xcd = blockIdx.x & 7u, lw = blockIdx.x >> 3;
    const unsigned q = ntiles >> 3, rem = ntiles & 7u;
    const unsigned begin = xcd * q + (xcd < rem ? xcd : rem);
    last = begin + q + (xcd < rem ? 1u : 0u);
    stride = (gridDim.x - xcd + 7u) >> 3;       // workgroups of this XCD
    first = begin + lw;
}

// The tile [C][xrows][XW] whose origin is image position (r_org, c_org) of image xi (C*H*W < 2^31
// elements), as a thread sees it: element e of the thread is flat index tid + 256 e.
struct TileGeom {
    const float *xi;
    int C, H, W, r_org, c_org, xrows, XR, XW;
};

// One element: where it comes from (clamped into the image), where it goes in LDS (-1: nowhere) and
// whether it lies inside the image.
// With DIR = 1 the tile lives in mirrored coordinates (rows, columns and channels reversed), which
// turns the transposed operator M^T into a causal convolution again; four consecutive mirrored
// columns are four consecutive image columns in reverse order.
template <bool vec, int DIR>
__device__ __forceinline__ void tile_elem(const TileGeom &g, unsigned raw, unsigned total, unsigned line, unsigned m_line,
                                          unsigned m_rows, unsigned &src, int &dst, bool &keep)
{
    constexpr int step = vec ? 4 : 1;
    const unsigned idx = raw < total ? raw : total - 1;
    const unsigned rr = fastdiv(idx, line, m_line), cq = idx - rr * line;
    const unsigned ch = fastdiv(rr, g.xrows, m_rows), r = rr - ch * g.xrows;
    const int gr = g.r_org + (int)r, gc = g.c_org + step * (int)cq;
    keep = gr >= 0 && gr < g.H && gc >= 0 && gc < g.W;
    const int grc = gr < 0 ? 0 : (gr >= g.H ? g.H - 1 : gr);
    const int gcc = gc < 0 ? 0 : (gc >= g.W ? g.W - step : gc);
    if (DIR)
        src = ((g.C - 1 - ch) * g.H + (g.H - 1 - grc)) * g.W + (g.W - step - gcc);
    else
        src = (ch * g.H + grc) * g.W + gcc;
    dst = raw < total ? (int)((ch * g.XR + r) * g.XW + step * cq) : -1;
}

// Tile loader: NB loads at a time with clamped addresses (no branch around a load); out-of-image
// elements are zeroed when the batch is written to LDS.  A batch is issued (conv_tile_issue) and later
// written (conv_tile_commit), so that the batches of two tiles can be in flight together.
template <int NB>
struct TileBatch {
    float4 val[NB];
    int dst[NB];
    bool keep[NB];
};

template <bool vec, int DIR, int NB>
__device__ __forceinline__ void conv_tile_issue(const TileGeom &g, unsigned base, TileBatch<NB> &b)
{
    const unsigned line = vec ? g.XW >> 2 : g.XW;       // elements (16 or 4 bytes) per tile row
    const unsigned total = g.C * g.xrows * line;
    const unsigned m_line = magic(line), m_rows = magic(g.xrows);
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        unsigned src;
        tile_elem<vec, DIR>(g, base + j * 256, total, line, m_line, m_rows, src, b.dst[j], b.keep[j]);
        if (vec)
            b.val[j] = *reinterpret_cast<const float4 *>(g.xi + src);
        else
            b.val[j].x = g.xi[src];
    }
}

template <bool vec, int DIR, int NB>
__device__ __forceinline__ void conv_tile_commit(float *sx, const TileBatch<NB> &b)
{
#pragma unroll
    for (int j = 0; j < NB; ++j)
        if (b.dst[j] >= 0) {
            const bool kp = b.keep[j];
            if (vec && DIR)
                *reinterpret_cast<float4 *>(sx + b.dst[j]) = make_float4(kp ? b.val[j].w : 0.f, kp ? b.val[j].z : 0.f,
                                                                          kp ? b.val[j].y : 0.f, kp ? b.val[j].x : 0.f);
            else if (vec)
                *reinterpret_cast<float4 *>(sx + b.dst[j]) = make_float4(kp ? b.val[j].x : 0.f, kp ? b.val[j].y : 0.f,
                                                                          kp ? b.val[j].z : 0.f, kp ? b.val[j].w : 0.f);
            else
                sx[b.dst[j]] = kp ? b.val[j].x : 0.f;
        }
}

template <bool vec, int DIR, int NB = kConvLoadBatch>
__device__ __forceinline__ void conv_load_tile(const TileGeom &g, float *sx)
{
    const unsigned line = vec ? g.XW >> 2 : g.XW;
    const unsigned total = g.C * g.xrows * line;
    for (unsigned base = threadIdx.x; base < total; base += NB * 256) {
        TileBatch<NB> b;
        conv_tile_issue<vec, DIR, NB>(g, base, b);
        conv_tile_commit<vec, DIR, NB>(sx, b);
    }
}

// loads in flight per thread for a tile of `elems` elements: all of them when that is fewer than kConvLoadBatch
constexpr int conv_batch_for(int elems) { return (elems + 255) / 256 < kConvLoadBatch ? (elems + 255) / 256 : kConvLoadBatch; }

// ---- few channels: lane = pixel ---------------------------------------------------------------
// Tile of kConvRows x TW pixels (TW = 32, 64 or 128), LDS tile [C][kConvRows + K - 1][TW + 4].
// A wave works on two batches of 64 pixels at a time (two independent accumulators); all LDS
// offsets of the taps are compile-time constants.
// DW (with DIR = 1, the backward pass of the convolution): the same walk over the tiles also forms the
// convolution's weight gradient, dw[o][i][a][b] = sum_p g[o][p] x2[i][p - d] with d = (K-1-a, K-1-b) (Eq. 1 is
// linear in w).  Seen from the x2 pixel q = p - d this is sum_q x2[i][q] g[o][q + d], and in the mirrored
// coordinates of this tile q + d lies up / left of q: exactly the halo the tile of g already has.  So only a
// halo-free tile of x2 is staged besides, and every 16 pixels cost ceil(C K K / 4) outer products
// (v_mfma_f32_4x4x1: rows = channels of x2, columns = shifted channels of g).  The workgroup keeps its sums
// over all its tiles in registers and writes one row of part[workgroup][C*C*K*K] at the end (un-negated,
// unmasked, true index order); x2 and g are read from memory once.
// CONV = false (with DW): only the weight-gradient sums are formed, y is not touched (the backward pass of the
// inverse convolution uses it with g = dL/dy and the sign of the second pass flipped, Theorem 2).
template <int C, int K, int TW, bool VEC, int DIR, bool DW = false, bool CONV = true>
__global__ __launch_bounds__(256) void k_conv_small(const float *__restrict__ x, const float *__restrict__ w,
                                                   float *__restrict__ y, int H, int W, int tiles_r, int tiles_c,
                                                   unsigned ntiles, const float *__restrict__ x2 = nullptr,
                                                   float *__restrict__ part = nullptr)
{
    static_assert(!DW || DIR == 1, "the weight gradient rides on the transposed convolution");
    constexpr int NCOL = C * K * K, NSW = (NCOL + 3) / 4, PW = C * NCOL;
    constexpr int HALO = 4;                      // K - 1 <= 4
    constexpr int XR = kConvRows + K - 1, XW = TW + HALO;
    constexpr int LW = TW < 64 ? TW : 64;        // pixels of one row a wave covers per batch
    constexpr int RPB = 64 / LW;                 // rows per batch
    constexpr int BPR = TW / LW;                 // batches per row
    constexpr int NBATCH = kConvRows * TW / 64;
    extern __shared__ float sx[];
    float *sx2 = sx + C * XR * XW;               // DW: [C][kConvRows][TW], no halo
    unsigned t0, t1, tstep;
    tile_sweep(ntiles, t0, t1, tstep);
    if (t0 >= t1) {
        if (DW)
            for (int e = threadIdx.x; e < PW; e += 256)
                part[(size_t)blockIdx.x * PW + e] = 0.0f;
        return;
    }
    f32x4 accw[DW ? NSW : 1];
    int woff[DW ? NSW : 1];
    if (DW) {
        const int j = threadIdx.x & 3;
#pragma unroll
        for (int s = 0; s < NSW; ++s) {
            accw[s] = f32x4{0.f, 0.f, 0.f, 0.f};
            const int col = (4 * s + j < NCOL) ? 4 * s + j : 0;       // column (o', da, db) in mirrored indices
            const int o = col / (K * K), da = (col / K) % K, db = col % K;
            woff[s] = (o * XR + (K - 1) - da) * XW + HALO - db;
        }
    }

    // A operands: a lane holds the weights of output channel o = lane % 4 (zero for o >= C and for
    // the masked entries of the current-pixel tap), gathered with one load per (i, tap)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, o_lane = lane & 3;
    const int oc = o_lane < C ? o_lane : 0;
    float wA[C][K][K];
#pragma unroll
    for (int i = 0; i < C; ++i)
#pragma unroll
        for (int a = 0; a < K; ++a)
#pragma unroll
            for (int b = 0; b < K; ++b) {
                const bool masked = (a == K - 1 && b == K - 1 && i > o_lane) || o_lane >= C;
                const int oo = DIR ? C - 1 - i : oc, ii = DIR ? C - 1 - oc : i;     // mirrored: transposed, reversed
                const float v = w[((oo * C + ii) * K + a) * K + b];
                wA[i][a][b] = masked ? 0.0f : v;
            }

    const unsigned m_tc = magic(tiles_c), m_tr = magic(tiles_r);
    auto geom = [&](unsigned t, size_t &n, int &r0, int &c0, int &rows) {
        const unsigned q = fastdiv(t, tiles_c, m_tc), tc = t - q * tiles_c;
        const unsigned img = fastdiv(q, tiles_r, m_tr), tr = q - img * tiles_r;
        n = img;
        r0 = tr * kConvRows;
        c0 = tc * TW;
        rows = (H - r0 < kConvRows) ? H - r0 : kConvRows;
        return TileGeom{x + n * C * H * W, C, H, W, r0 - (K - 1), c0 - HALO, rows + K - 1, XR, XW};
    };

    size_t n;
    int r0, c0, rows;
    const int lr = lane / LW, lc = lane % LW;
    constexpr int E1 = C * XR * (VEC ? XW / 4 : XW), E2 = C * kConvRows * (VEC ? TW / 4 : TW);
    constexpr int NB1 = conv_batch_for(E1), NB2 = conv_batch_for(E2);
    // Small tiles with the weight gradient: both tiles are one batch of loads each, issued together, and the
    // next tile's batches are issued before this tile's products, so that they are in flight meanwhile.
    constexpr bool kAhead2 = DW && E1 <= 256 * NB1 && E2 <= 256 * NB2 && NB1 + NB2 <= 12;
    TileBatch<kAhead2 ? NB1 : 1> b1;
    TileBatch<kAhead2 ? NB2 : 1> b2;
    auto issue_both = [&](unsigned t) {
        if constexpr (kAhead2) {
            size_t nn;
            int rr0, cc0, rrows;
            const TileGeom g = geom(t, nn, rr0, cc0, rrows);
            const TileGeom g2{x2 + nn * C * H * W, C, H, W, rr0, cc0, rrows, kConvRows, TW};
            conv_tile_issue<VEC, DIR, NB1>(g, threadIdx.x, b1);
            conv_tile_issue<VEC, DIR, NB2>(g2, threadIdx.x, b2);
        }
    };
    issue_both(t0);
    for (unsigned t = t0; t < t1; t += tstep) {
        const TileGeom g = geom(t, n, r0, c0, rows);
        if constexpr (kAhead2) {
            conv_tile_commit<VEC, DIR, NB1>(sx, b1);
            conv_tile_commit<VEC, DIR, NB2>(sx2, b2);
            if (t + tstep < t1)
                issue_both(t + tstep);
        } else {
            conv_load_tile<VEC, DIR, NB1>(g, sx);
            if (DW) {
                const TileGeom g2{x2 + n * C * H * W, C, H, W, r0, c0, rows, kConvRows, TW};
                conv_load_tile<VEC, DIR, NB2>(g2, sx2);
            }
        }
        __syncthreads();
        float *__restrict__ yi = y + n * C * H * W;
        for (int bi = 2 * wave; CONV && bi < NBATCH; bi += 8) {
            // batches bi and bi + 1
            const int pr0 = (bi / BPR) * RPB + lr, pc0 = (bi % BPR) * LW + lc;
            constexpr int D1 = (BPR == 2) ? 64 : RPB * XW;     // LDS distance between the two batches
            const int pr1 = (BPR == 2) ? pr0 : pr0 + RPB, pc1 = (BPR == 2) ? pc0 + 64 : pc0;
            if ((bi / BPR) * RPB >= rows)
                break;
            const float *bp = sx + pr0 * XW + pc0 + HALO - (K - 1);
            f32x4 acc0 = f32x4{0.f, 0.f, 0.f, 0.f}, acc1 = f32x4{0.f, 0.f, 0.f, 0.f};
            // step s = (i, a, b); the x values are read kAhead steps ahead of their use
            constexpr int NSTEP = C * K * K, kAhead = 6;
            float bv[kAhead + 1][2];
#pragma unroll
            for (int s = 0; s < kAhead && s < NSTEP; ++s) {
                const int off = ((s / (K * K)) * XR + (s / K) % K) * XW + s % K;
                bv[s][0] = bp[off];
                bv[s][1] = bp[off + D1];
            }
#pragma unroll
            for (int s = 0; s < NSTEP; ++s) {
                if (s + kAhead < NSTEP) {
                    const int s2 = s + kAhead;
                    const int off = ((s2 / (K * K)) * XR + (s2 / K) % K) * XW + s2 % K;
                    bv[s2 % (kAhead + 1)][0] = bp[off];
                    bv[s2 % (kAhead + 1)][1] = bp[off + D1];
                }
                __builtin_amdgcn_sched_barrier(0);      // keep the reads ahead of the instructions below
                const float wv = wA[s / (K * K)][(s / K) % K][s % K];
                acc0 = __builtin_amdgcn_mfma_f32_4x4x1f32(wv, bv[s % (kAhead + 1)][0], acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_4x4x1f32(wv, bv[s % (kAhead + 1)][1], acc1, 0, 0, 0);
            }
            if (pr0 < rows && c0 + pc0 < W) {
                const unsigned off = DIR ? (H - 1 - r0 - pr0) * W + (W - 1 - c0 - pc0) : (r0 + pr0) * W + c0 + pc0;
#pragma unroll
                for (int o = 0; o < C; ++o)
                    yi[off + (DIR ? C - 1 - o : o) * H * W] = acc0[o];
            }
            if (pr1 < rows && c0 + pc1 < W) {
                const unsigned off = DIR ? (H - 1 - r0 - pr1) * W + (W - 1 - c0 - pc1) : (r0 + pr1) * W + c0 + pc1;
#pragma unroll
                for (int o = 0; o < C; ++o)
                    yi[off + (DIR ? C - 1 - o : o) * H * W] = acc1[o];
            }
        }
        if (DW) {
            // lane = (block b, j): row i' = j of x2, column 4s + j of the shifted g; block b takes pixel 16 grp + b
            // of a tile row (pixels outside the image are zeros in the x2 tile and contribute nothing)
            const int j = lane & 3, b = lane >> 2;
            const float *ap = sx2 + (j < C ? j : 0) * kConvRows * TW + b;
            for (int pr = wave; pr < rows; pr += 4) {
                const float *bp = sx + pr * XW + b;
#pragma unroll
                for (int grp = 0; grp < TW / 16; ++grp) {
                    const float av = ap[pr * TW + 16 * grp];
                    float bv[NSW];
#pragma unroll
                    for (int s = 0; s < NSW; ++s)
                        bv[s] = bp[woff[s] + 16 * grp];
#pragma unroll
                    for (int s = 0; s < NSW; ++s)
                        accw[s] = __builtin_amdgcn_mfma_f32_4x4x1f32(av, bv[s], accw[s], 0, 0, 0);
                }
            }
        }
        __syncthreads();        // the tile is overwritten next
    }
    if (DW) {
        // fixed-order sum over the 16 blocks of each wave, then over the four waves; lane (b, j) register
        // (s, i') holds block b's sum of entry (i', column 4s + j)
        float *sred = sx;                               // [256][NSW*4], then [4][PW]
        float *swave = sred + 256 * NSW * 4;
#pragma unroll
        for (int s = 0; s < NSW; ++s)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                sred[threadIdx.x * (NSW * 4) + s * 4 + i] = accw[s][i];
        __syncthreads();
        for (int idx = threadIdx.x; idx < 4 * PW; idx += 256) {
            const int e = idx % PW, wv = idx / PW;
            const int ip = e / NCOL, col = e % NCOL;            // mirrored x2 channel i', column (o', da, db)
            const int s = col >> 2, jj = col & 3;
            float sum = 0.0f;
#pragma unroll
            for (int bb = 0; bb < 16; ++bb)
                sum += sred[(wv * 64 + bb * 4 + jj) * (NSW * 4) + s * 4 + ip];
            swave[wv * PW + e] = sum;
        }
        __syncthreads();
        for (int e = threadIdx.x; e < PW; e += 256) {
            const int ip = e / NCOL, col = e % NCOL;
            const int op = col / (K * K), da = (col / K) % K, db = col % K;
            // mirrored channel c' is true channel C-1-c'; reach (da, db) is tap (K-1-da, K-1-db)
            const int dst = (((C - 1 - op) * C + (C - 1 - ip)) * K + (K - 1 - da)) * K + (K - 1 - db);
            part[(size_t)blockIdx.x * PW + dst] = ((swave[e] + swave[PW + e]) + swave[2 * PW + e]) + swave[3 * PW + e];
        }
    }
}

// ---- any channel count: M = 16 pixels, N = 16 output channels, K = (input channel, tap) --------
// Tile of TR x 64 pixels (TR = 16 unless LDS forces fewer rows).  Instruction s of the contraction
// covers pairs kk = 4s + g (g = lane / 16): A[pixel][g] = x at that pair, B[g][n] = w[o = 16 ob + n][pair kk],
// so a lane ends up with four consecutive pixels of one output channel and stores them as 16 bytes.  The A operands and the LDS offsets of the pairs are tabulated in LDS once per
// workgroup and held in registers NSC instructions at a time; a wave forms the four 16-pixel groups
// of one tile row together (four independent accumulators).
template <int NSC, bool VEC, int DIR>
__global__ __launch_bounds__(256, 2) void k_conv_mfma16(const float *__restrict__ x, const float *__restrict__ w,
                                                    float *__restrict__ y, int C, int H, int W, int k, int halo,
                                                    int TR, int tiles_r, int tiles_c, int nck, unsigned ntiles)
{
    constexpr int TW = 64;
    extern __shared__ float smem[];
    const int XR = TR + k - 1, XW = TW + halo;
    const int NS = nck * NSC, OB = (C + 15) >> 4, NK = C * k * k;
    float *sx = smem;                                   // [C][XR][XW]
    float *sA = sx + C * XR * XW;                       // [OB][NS][64]
    int *sOff = reinterpret_cast<int *>(sA + OB * NS * 64);    // [NS][4]
    unsigned t0, t1, tstep;
    tile_sweep(ntiles, t0, t1, tstep);
    if (t0 >= t1)
        return;

    const unsigned m_tc = magic(tiles_c), m_tr = magic(tiles_r);
    auto geom = [&](unsigned t, size_t &n, int &r0, int &c0, int &rows) {
        const unsigned q = fastdiv(t, tiles_c, m_tc), tc = t - q * tiles_c;
        const unsigned img = fastdiv(q, tiles_r, m_tr), tr = q - img * tiles_r;
        n = img;
        r0 = tr * TR;
        c0 = tc * TW;
        rows = (H - r0 < TR) ? H - r0 : TR;
        return TileGeom{x + n * C * H * W, C, H, W, r0 - (k - 1), c0 - halo, rows + k - 1, XR, XW};
    };
    size_t n;
    int r0, c0, rows;
    {
        // a thread fills the table entries of its own lane for instructions s = wave, wave + 4, ...;
        // the loads of kTab instructions are issued together, masking is applied afterwards
        constexpr int kTab = 8;
        const unsigned kk2 = k * k, m_kk = magic(kk2), m_k = magic(k);
        const unsigned l = threadIdx.x & 63;
        for (int ob = 0; ob < OB; ++ob) {
            const unsigned o = 16 * ob + (l & 15), oc = o < (unsigned)C ? o : 0;
            for (int s0 = threadIdx.x >> 6; s0 < NS; s0 += 4 * kTab) {
                float val[kTab];
                bool keep[kTab];
#pragma unroll
                for (int j = 0; j < kTab; ++j) {
                    const unsigned kk = 4 * (s0 + 4 * j) + (l >> 4);
                    const unsigned kc = kk < (unsigned)NK ? kk : 0;    // padding pairs: zero weights, any valid offset
                    const unsigned i = fastdiv(kc, kk2, m_kk), t = kc - i * kk2;
                    const unsigned a = fastdiv(t, k, m_k), b = t - a * k;
                    const unsigned oo = DIR ? C - 1 - i : oc, ii = DIR ? C - 1 - oc : i;    // mirrored: transposed, reversed
                    val[j] = w[(oo * C + ii) * kk2 + t];
                    keep[j] = kk < (unsigned)NK && o < (unsigned)C && !(t == kk2 - 1 && i > o);
                    if (ob == 0 && (l & 15) == 0 && s0 + 4 * j < NS)
                        sOff[kk] = (i * XR + a) * XW + b + halo - (k - 1);
                }
#pragma unroll
                for (int j = 0; j < kTab; ++j)
                    if (s0 + 4 * j < NS)
                        sA[(ob * NS + s0 + 4 * j) * 64 + l] = keep[j] ? val[j] : 0.0f;
            }
        }
    }

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nn = lane & 15, g4 = lane >> 4;
    float wA[NSC];
    int boff[NSC];
    for (unsigned t = t0; t < t1; t += tstep) {
        const TileGeom g = geom(t, n, r0, c0, rows);
        conv_load_tile<VEC, DIR>(g, sx);
        __syncthreads();        // also orders the tables before their first use
        float *__restrict__ yi = y + n * C * H * W;
        for (int ob = 0; ob < OB; ++ob) {
            if (nck == 1 && (OB > 1 || t == t0)) {
#pragma unroll
                for (int s = 0; s < NSC; ++s) {
                    wA[s] = sA[(ob * NS + s) * 64 + lane];
                    boff[s] = sOff[4 * s + g4];
                }
            }
            for (int pr = wave; pr < rows; pr += 4) {
                f32x4 acc[4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    acc[u] = f32x4{0.f, 0.f, 0.f, 0.f};
                const float *bp = sx + pr * XW + nn;
                for (int ck = 0; ck < nck; ++ck) {
                    if (nck > 1) {
#pragma unroll
                        for (int s = 0; s < NSC; ++s) {
                            wA[s] = sA[(ob * NS + ck * NSC + s) * 64 + lane];
                            boff[s] = sOff[4 * (ck * NSC + s) + g4];
                        }
                    }
                    // B operands are read kAhead instructions ahead of their use
                    constexpr int kAhead = 2;
                    float bv[kAhead + 1][4];
#pragma unroll
                    for (int s = 0; s < kAhead && s < NSC; ++s)
#pragma unroll
                        for (int u = 0; u < 4; ++u)
                            bv[s][u] = bp[boff[s] + 16 * u];
#pragma unroll
                    for (int s = 0; s < NSC; ++s) {
                        if (s + kAhead < NSC) {
#pragma unroll
                            for (int u = 0; u < 4; ++u)
                                bv[(s + kAhead) % (kAhead + 1)][u] = bp[boff[s + kAhead] + 16 * u];
                        }
                        __builtin_amdgcn_sched_barrier(0);      // keep the reads ahead of the instructions below
#pragma unroll
                        for (int u = 0; u < 4; ++u)
                            acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(bv[s % (kAhead + 1)][u], wA[s], acc[u], 0, 0, 0);
                    }
                }
                // lane (nn, g4) register j holds output channel 16 ob + nn of pixel 16u + 4 g4 + j
                const int o = 16 * ob + nn;
                if (o < C) {
                    // mirrored: pixel (row, c .. c+3) is image pixel (H-1-row, W-1-c-3 .. W-1-c) of channel C-1-o
                    const int row = r0 + pr;
                    float *yo = DIR ? yi + ((C - 1 - o) * H + (H - 1 - row)) * W : yi + (o * H + row) * W;
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int c = c0 + 16 * u + 4 * g4;
                        if (VEC) {
                            if (c < W) {
                                if (DIR)
                                    *reinterpret_cast<float4 *>(yo + W - 4 - c) =
                                        make_float4(acc[u][3], acc[u][2], acc[u][1], acc[u][0]);
                                else
                                    *reinterpret_cast<float4 *>(yo + c) = make_float4(acc[u][0], acc[u][1], acc[u][2], acc[u][3]);
                            }
                        } else {
#pragma unroll
                            for (int j = 0; j < 4; ++j)
                                if (c + j < W)
                                    yo[DIR ? W - 1 - c - j : c + j] = acc[u][j];
                        }
                    }
                }
            }
        }
        __syncthreads();        // the tile is overwritten next
    }
}

// ---- any shape: one thread per output element ---------------------------------------------------
template <int DIR>
__global__ __launch_bounds__(256) void k_conv_generic(const float *__restrict__ x, const float *__restrict__ w,
                                                     float *__restrict__ y, int B, int C, int H, int W, int k)
{
    const size_t total = (size_t)B * C * H * W;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
        const int c = (int)(idx % W), r = (int)((idx / W) % H), o = (int)((idx / ((size_t)W * H)) % C);
        const size_t n = idx / ((size_t)W * H * C);
        float acc = 0.0f;
        for (int i = 0; i < C; ++i)
            for (int a = 0; a < k; ++a) {
                const int rr = r - (k - 1) + a;
                if (rr < 0)
                    continue;
                for (int b = 0; b < k; ++b) {
                    const int cc = c - (k - 1) + b;
                    if (cc >= 0)
                        acc += weff<DIR>(w, C, k, o, i, a, b) * x[gidx<DIR>((int)n, i, rr, cc, C, H, W)];
                }
            }
        y[gidx<DIR>((int)n, o, r, c, C, H, W)] = acc;
    }
}

static unsigned conv_grid(size_t ntiles)
{
    return ntiles < (size_t)kConvMaxGrid ? (unsigned)ntiles : (unsigned)kConvMaxGrid;
}

template <int C, int K, int TW, int DIR>
static void launch_small_tw(const float *x, const float *w, float *y, int B, int H, int W, int vec, hipStream_t stream)
{
    const int tiles_r = (H + kConvRows - 1) / kConvRows, tiles_c = (W + TW - 1) / TW;
    const size_t ntiles = (size_t)B * tiles_r * tiles_c;
    const size_t lds = sizeof(float) * C * (kConvRows + K - 1) * (TW + 4);
    const unsigned grid = conv_grid(ntiles);
    if (vec)
        hipLaunchKernelGGL((k_conv_small<C, K, TW, true, DIR>), dim3(grid), dim3(256), lds, stream, x, w, y, H, W,
                           tiles_r, tiles_c, (unsigned)ntiles);
    else
        hipLaunchKernelGGL((k_conv_small<C, K, TW, false, DIR>), dim3(grid), dim3(256), lds, stream, x, w, y, H, W,
                           tiles_r, tiles_c, (unsigned)ntiles);
}

// LDS of the backward form: the tile of g with halo, the tile of x2 without; the final reduction reuses them
template <int C, int K, int TW>
static size_t conv_small_dw_lds()
{
    constexpr size_t ncol = (size_t)C * K * K, nsw = (ncol + 3) / 4;
    const size_t tiles = (size_t)C * (kConvRows + K - 1) * (TW + 4) + (size_t)C * kConvRows * TW;
    const size_t red = 256 * nsw * 4 + 4 * (size_t)C * ncol;
    return sizeof(float) * (tiles > red ? tiles : red);
}

template <int C, int K, int TW>
static unsigned launch_small_dw_tw(const float *g, const float *w, float *dx, const float *x2, float *part, int B, int H,
                                   int W, hipStream_t stream)
{
    const int tiles_r = (H + kConvRows - 1) / kConvRows, tiles_c = (W + TW - 1) / TW;
    const size_t ntiles = (size_t)B * tiles_r * tiles_c;
    const size_t lds = conv_small_dw_lds<C, K, TW>();
    unsigned grid = conv_grid(ntiles);
    if (!dx) {
        // as many workgroups as are resident at once (registers and LDS: five per compute unit for 3 channels),
        // so that no second, partly filled round of workgroups follows the first
        const void *fn = reinterpret_cast<const void *>(&k_conv_small<C, K, TW, true, 1, true, false>);
        if (!ensure_dynamic_lds(fn, lds))
            return 0;
        const int resident = resident_workgroups(fn, 256, lds);
        const size_t cap = resident > 0 && resident < kConvMaxGridDw ? (size_t)resident : (size_t)kConvMaxGridDw;
        grid = ntiles < cap ? (unsigned)ntiles : (unsigned)cap;
    }
    if (dx) {
        if (!ensure_dynamic_lds(reinterpret_cast<const void *>(&k_conv_small<C, K, TW, true, 1, true>), lds))
            return 0;
        hipLaunchKernelGGL((k_conv_small<C, K, TW, true, 1, true>), dim3(grid), dim3(256), lds, stream, g, w, dx, H, W,
                           tiles_r, tiles_c, (unsigned)ntiles, x2, part);
    } else {        // weight-gradient sums only
        if (!ensure_dynamic_lds(reinterpret_cast<const void *>(&k_conv_small<C, K, TW, true, 1, true, false>), lds))
            return 0;
        hipLaunchKernelGGL((k_conv_small<C, K, TW, true, 1, true, false>), dim3(grid), dim3(256), lds, stream, g, w, dx,
                           H, W, tiles_r, tiles_c, (unsigned)ntiles, x2, part);
    }
    return grid;
}

template <int C, int K>
static unsigned launch_small_dw(const float *g, const float *w, float *dx, const float *x2, float *part, int B, int H,
                                int W, hipStream_t stream)
{
    if (W <= 32)
        return launch_small_dw_tw<C, K, 32>(g, w, dx, x2, part, B, H, W, stream);
    if (W <= 64)
        return launch_small_dw_tw<C, K, 64>(g, w, dx, x2, part, B, H, W, stream);
    return launch_small_dw_tw<C, K, 128>(g, w, dx, x2, part, B, H, W, stream);
}

template <int C, int K, int DIR>
static void launch_small(const float *x, const float *w, float *y, int B, int H, int W, int vec, hipStream_t stream)
{
    if (W <= 32)
        launch_small_tw<C, K, 32, DIR>(x, w, y, B, H, W, vec, stream);
    else if (W <= 64)
        launch_small_tw<C, K, 64, DIR>(x, w, y, B, H, W, vec, stream);
    else
        launch_small_tw<C, K, 128, DIR>(x, w, y, B, H, W, vec, stream);
}

// Plan of the 16-channel kernel: instructions per register chunk, chunks, halo columns, tile rows,
// LDS bytes (0: does not fit).
struct ConvPlan {
    int nsc, nck, halo, tr;
    size_t lds;
};

static ConvPlan plan_m16(int C, int k)
{
    ConvPlan p{};
    const int ns = (C * k * k + 3) / 4, ob = (C + 15) / 16;
    p.nsc = ns <= 40 ? 4 * ((ns + 3) / 4) : 32;
    p.nck = (ns + p.nsc - 1) / p.nsc;
    p.halo = 4 * ((k - 1 + 3) / 4);
    if (p.halo == 0)
        p.halo = 4;
    const size_t tables = sizeof(float) * ob * p.nck * p.nsc * 64 + sizeof(int) * p.nck * p.nsc * 4;
    for (p.tr = kConvRows; p.tr >= 1; --p.tr) {
        const size_t tile = sizeof(float) * C * (p.tr + k - 1) * (64 + p.halo);
        p.lds = tile + tables;
        if (p.lds <= kConvLdsBudget)
            return p;
    }
    p.lds = 0;
    return p;
}

template <int NSC, int DIR>
static void launch_m16(const float *x, const float *w, float *y, int B, int C, int H, int W, int k, const ConvPlan &p,
                       int vec, hipStream_t stream)
{
    const int tiles_r = (H + p.tr - 1) / p.tr, tiles_c = (W + 63) / 64;
    const size_t ntiles = (size_t)B * tiles_r * tiles_c;
    const unsigned grid = conv_grid(ntiles);
    if (vec)
        hipLaunchKernelGGL((k_conv_mfma16<NSC, true, DIR>), dim3(grid), dim3(256), p.lds, stream, x, w, y, C, H, W, k,
                           p.halo, p.tr, tiles_r, tiles_c, p.nck, (unsigned)ntiles);
    else
        hipLaunchKernelGGL((k_conv_mfma16<NSC, false, DIR>), dim3(grid), dim3(256), p.lds, stream, x, w, y, C, H, W, k,
                           p.halo, p.tr, tiles_r, tiles_c, p.nck, (unsigned)ntiles);
}

// y = M x (DIR = 0) or y = M^T x (DIR = 1, the same kernels in mirrored coordinates).
template <int DIR>
static int launch_conv_dir(const float *x, const float *w, float *y, int B, int C, int H, int W, int k,
                           hipStream_t stream)
{
    const int vec = (W % 4) == 0 && (((size_t)x | (size_t)y) & 15) == 0;
    const size_t tiles = (size_t)B * H * ((W + 63) / 64);   // upper bound of the tile count
    bool done = true;
    if (tiles > 0x7fffffffull || (size_t)C * H * W > 0x7fffffffull) done = false;
    else if (C == 1 && k == 3) launch_small<1, 3, DIR>(x, w, y, B, H, W, vec, stream);
    else if (C == 2 && k == 3) launch_small<2, 3, DIR>(x, w, y, B, H, W, vec, stream);
    else if (C == 3 && k == 3) launch_small<3, 3, DIR>(x, w, y, B, H, W, vec, stream);
    else if (C == 4 && k == 3) launch_small<4, 3, DIR>(x, w, y, B, H, W, vec, stream);
    else if (C == 3 && k == 5) launch_small<3, 5, DIR>(x, w, y, B, H, W, vec, stream);
    else {
        const ConvPlan p = plan_m16(C, k);
        if (p.lds == 0) done = false;
        else switch (p.nsc) {
            case 4: launch_m16<4, DIR>(x, w, y, B, C, H, W, k, p, vec, stream); break;
            case 8: launch_m16<8, DIR>(x, w, y, B, C, H, W, k, p, vec, stream); break;
            case 12: launch_m16<12, DIR>(x, w, y, B, C, H, W, k, p, vec, stream); break;
            case 16: launch_m16<16, DIR>(x, w, y, B, C, H, W, k, p, vec, stream); break;
            case 20: launch_m16<20, DIR>(x, w, y, B, C, H, W, k, p, vec, stream); break;
            case 24: launch_m16<24, DIR>(x, w, y, B, C, H, W, k, p, vec, stream); break;
            case 28: launch_m16<28, DIR>(x, w, y, B, C, H, W, k, p, vec, stream); break;
            case 32: launch_m16<32, DIR>(x, w, y, B, C, H, W, k, p, vec, stream); break;
            case 36: launch_m16<36, DIR>(x, w, y, B, C, H, W, k, p, vec, stream); break;
            default: launch_m16<40, DIR>(x, w, y, B, C, H, W, k, p, vec, stream); break;
        }
    }
    if (!done) {
        const size_t total = (size_t)B * C * H * W;
        size_t blocks = (total + 255) / 256;
        if (blocks > 65536) blocks = 65536;
        hipLaunchKernelGGL(k_conv_generic<DIR>, dim3((unsigned)blocks), dim3(256), 0, stream, x, w, y, B, C, H, W, k);
    }
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

// Few channels, rows of whole 16-byte pieces: dL/dx = M^T g and the partial sums of dL/dw in one pass over g
// and x.  part needs conv_bwd_fused_rows() rows of C*C*k*k floats.
bool conv_bwd_fused_supported(int C, int H, int W, int k)
{
    return ((C >= 1 && C <= 4 && k == 3) || (C == 3 && k == 5)) && (W % 4) == 0 && (size_t)C * H * W <= 0x7fffffffull;
}

size_t conv_bwd_fused_rows() { return kConvMaxGridDw; }

// dx may be null: then only the partial sums of the weight gradient are formed (g and x read once).
// Returns the number of partial rows written (0: not launched)
int launch_conv_bwd_fused(const float *g, const float *w, float *dx, const float *x, float *part, int B, int C, int H,
                          int W, int k, hipStream_t stream, unsigned *rows)
{
    unsigned n = 0;
    if (C == 1 && k == 3) n = launch_small_dw<1, 3>(g, w, dx, x, part, B, H, W, stream);
    else if (C == 2 && k == 3) n = launch_small_dw<2, 3>(g, w, dx, x, part, B, H, W, stream);
    else if (C == 3 && k == 3) n = launch_small_dw<3, 3>(g, w, dx, x, part, B, H, W, stream);
    else if (C == 4 && k == 3) n = launch_small_dw<4, 3>(g, w, dx, x, part, B, H, W, stream);
    else if (C == 3 && k == 5) n = launch_small_dw<3, 5>(g, w, dx, x, part, B, H, W, stream);
    *rows = n;
    if (!n)
        return INVCONV_ERR_UNSUPPORTED;
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

int launch_conv(int dir, const float *x, const float *w, float *y, int B, int C, int H, int W, int k, hipStream_t stream)
{
    return dir ? launch_conv_dir<1>(x, w, y, B, C, H, W, k, stream) : launch_conv_dir<0>(x, w, y, B, C, H, W, k, stream);
}

}  // namespace invconv
