// Weight gradient on the matrix cores for C <= 16 (Eq. 4 with Theorem 2):
//   dw[o][i][a][b] = - sum_{n,r,c} v[n][o][r][c] * x[n][i][r-(k-1)+a][c-(k-1)+b]
// is a GEMM with M = C output channels, N = C*k*k "shifted x" columns and the
// pixels of the whole batch as the contraction index.  gfx950 only.
//
// Pass 1: one workgroup (4 waves) per (image, chunk of RT rows).  v and x (with
// a zero halo of k-1 rows/columns on the top/left) are staged in LDS.  Each
// v_mfma_f32_16x16x4_f32 contracts 4 pixels: A[m][kk] = v[o = m][pixel 4q+kk],
// B[kk][nn] = column 16s+nn of pixel 4q+kk, result D_s[m][nn].  Rows m >= C and
// columns >= C*k*k are padding: they read valid data and are never written out.
// The four waves take pixel groups round robin and are added in wave order
// through LDS; the un-negated partial sums go to part[workgroup][P].
// A workgroup takes a contiguous range of row chunks.  In the streaming mode (16-byte aligned rows,
// RT >= k-1) it reads every element of x and v once: the halo rows of a chunk are the last rows of
// the chunk before, kept in registers, and the next chunk is fetched into registers while the
// matrix cores work on the current one.
// Pass 2 (k_dw_reduce in the generic file) adds the rows of `part` in a fixed order.
#include "invconv_common.h"
#include "invconv_launch.h"

namespace invconv {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// Pointers of up to kChainMaxLayers independent (x, v) pairs handled by one launch.
struct DwBatch {
    const float *x[kChainMaxLayers];
    const float *v[kChainMaxLayers];
    // blocks of a result with more than 16 channels as the "layers" of one launch: channels of the x block and
    // of the v block of entry l (0: the launch's C and Cv)
    unsigned char cx[kChainMaxLayers];
    unsigned char cv[kChainMaxLayers];
};

// left halo of the x tile, in columns: at least k-1, a multiple of 4 (keeps rows 16-byte aligned)
__host__ __device__ constexpr int dw_halo(int k) { return k <= 5 ? 4 : ((k - 1 + 3) / 4) * 4; }
constexpr int kDwUnroll = 4;    // pixel quads per trip of the product loop
constexpr int kDwPre = 6;       // streaming mode: 16-byte pieces of each tile a thread holds in registers
constexpr size_t kDwStreamLdsBudget = 72 * 1024;   // streaming mode: two workgroups per compute unit

// More than 16 channels: the launcher cuts the C x C k k result into blocks of at most 16 x 16 k k and calls
// this kernel once per block with the tensors' base pointers moved to the block's first channels: C is then
// the number of x channels (columns / k k) of the block, Cv the number of v channels (rows), Ctot the
// channel count of the tensors (image stride).
template <int NS>
__global__ __launch_bounds__(256) void k_dw_partial_mfma(DwBatch batch, float *__restrict__ part, int B, int C,
                                                        int H, int W, int k, int RT, int nchunks, int G, int vec,
                                                        int XW, int SXC, int SVC, int Cv, int Ctot, int pstride,
                                                        int ipw, int Btot)
{
    extern __shared__ float smem[];
    // blockIdx = ((layer * B + n) * G + cg); this workgroup takes chunks cg, cg+G, ... of image n.
    // ipw > 1 (images of a single chunk, G = 1): B counts groups of ipw images and the workgroup takes the images
    // n ipw .. of the Btot there are, one after the other, into the same accumulators - one partial row per group
    // instead of one per image (1024 images of 48 x 8 x 8 wrote and re-read 85 MB of partial sums)
    const int cg = blockIdx.x % G, n = (blockIdx.x / G) % B, layer = blockIdx.x / (G * B);
    if (batch.cx[layer]) {      // a block of a larger result: its own channel counts (tiles are laid out for the launch's)
        C = batch.cx[layer];
        Cv = batch.cv[layer];
    }
    const float *__restrict__ x = batch.x[layer];
    const float *__restrict__ v = batch.v[layer];
    // XW >= W + halo, SXC >= (RT + k - 1) * XW and SVC >= RT * W: row / channel strides padded by the
    // host so that the 64 lanes of an operand read fall into different LDS banks
    const int NCOL = C * k * k;
    const int P = Cv * NCOL;
    const int CM = Cv > C ? Cv : C;
    float *sv = smem;                 // [Cv] x SVC, rows of W floats
    float *sx = sv + CM * SVC;        // [C] x SXC, rows of XW floats, origin at (r0-(k-1), -halo)
    const int halo = dw_halo(k);
    float *sred = smem;               // [4 waves][64 lanes][NS*4], reuses the tiles afterwards
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;

    const int nn = lane & 15, kk = lane >> 4;
    const int aoff = (nn < Cv ? nn : 0) * SVC;              // A row m = nn -> v[o = m]
    int boff[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const int col = (16 * s + nn < NCOL) ? 16 * s + nn : 0;
        const int i = col / (k * k), a = (col / k) % k, b = col % k;
        boff[s] = i * SXC + a * XW + b + halo - (k - 1);
    }
    f32x4 acc[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s)
        acc[s] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int cpw = (nchunks + G - 1) / G;          // chunks cg*cpw .. of image n, contiguous
    const int c_begin = cg * cpw, c_end = (c_begin + cpw < nchunks) ? c_begin + cpw : nchunks;
    const size_t img_stride = (size_t)Ctot * H * W;
    const int n_first = ipw > 1 ? n * ipw : n;
    const int trips = ipw > 1 ? (Btot - n_first < ipw ? Btot - n_first : ipw) : c_end - c_begin;
    size_t img = (size_t)n_first * img_stride;

    // streaming mode: this thread's pieces of a chunk (loop invariant): piece i is float4 c4 of row r of channel ch
    float4 pv[kDwPre], px[kDwPre], ph[kDwPre];
    int p_go[kDwPre], p_vl[kDwPre], p_xl[kDwPre], p_r[kDwPre];
    bool p_hv[kDwPre], p_hx[kDwPre];        // the piece's channel exists in the v / x block
    if (vec == 2) {
        const int W4 = W / 4;
#pragma unroll
        for (int i = 0; i < kDwPre; ++i) {
            const int idx = tid + 256 * i;
            const bool ok = idx < CM * RT * W4;
            const int c4 = idx % W4, rr = idx / W4;
            const int ch = ok ? rr / RT : 0, r = ok ? rr - ch * RT : 0;
            p_hv[i] = ok && ch < Cv;
            p_hx[i] = ok && ch < C;
            p_r[i] = ok ? r : -1;
            p_go[i] = (ch * H + r) * W + 4 * c4;
            p_vl[i] = ch * SVC + r * W + 4 * c4;
            p_xl[i] = ch * SXC + (r + k - 1) * XW + 4 * c4 + halo;
            pv[i] = px[i] = ph[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
        // the halo columns stay zero for the whole launch
        const int H4 = halo / 4;
        for (int idx = tid; idx < C * (RT + k - 1) * H4; idx += 256) {
            const int q = idx % H4, rr = idx / H4;
            const int ch = rr / (RT + k - 1), r = rr - ch * (RT + k - 1);
            *reinterpret_cast<float4 *>(sx + ch * SXC + r * XW + 4 * q) = make_float4(0.f, 0.f, 0.f, 0.f);
        }
        // rows above the first chunk, as if left by a chunk before it; then the first chunk itself
        const int rb = c_begin * RT;
#pragma unroll
        for (int i = 0; i < kDwPre; ++i) {
            const int r = p_r[i];
            if (p_hx[i] && r >= RT - (k - 1) && rb - RT + r >= 0 && c_begin < c_end)
                ph[i] = *reinterpret_cast<const float4 *>(x + img + p_go[i] + (ptrdiff_t)(rb - RT) * W);
            if (r >= 0 && rb + r < H && c_begin < c_end) {
                if (p_hv[i])
                    pv[i] = *reinterpret_cast<const float4 *>(v + img + p_go[i] + (size_t)rb * W);
                if (p_hx[i])
                    px[i] = *reinterpret_cast<const float4 *>(x + img + p_go[i] + (size_t)rb * W);
            }
        }
    }

    for (int it = 0; it < trips; ++it) {
        const int chunk = ipw > 1 ? 0 : c_begin + it;
        const int r0 = chunk * RT;
        const int rows = (H - r0 < RT) ? H - r0 : RT;
        const int xrows = rows + k - 1;
        __syncthreads();        // previous chunk's products are done with the tiles
        if (vec == 2) {
#pragma unroll
            for (int i = 0; i < kDwPre; ++i) {
                const int r = p_r[i];
                if (r >= 0) {
                    if (p_hv[i])
                        *reinterpret_cast<float4 *>(sv + p_vl[i]) = pv[i];
                    if (p_hx[i]) {
                        *reinterpret_cast<float4 *>(sx + p_xl[i]) = px[i];
                        if (r >= RT - (k - 1))      // last rows of the chunk before: rows 0 .. k-2 of the tile
                            *reinterpret_cast<float4 *>(sx + p_xl[i] - RT * XW) = ph[i];
                    }
                    if (ipw <= 1)
                        ph[i] = px[i];      // (single-chunk images: nothing above the chunk, ph stays zero)
                }
            }
        } else if (vec) {
            const int W4 = W / 4;
            for (int idx = tid; idx < Cv * rows * W4; idx += 256) {
                const int c4 = idx % W4, rr = idx / W4;         // rr = ch*rows + r
                const int ch = rr / rows, r = rr - ch * rows;
                const float4 val = *reinterpret_cast<const float4 *>(
                    v + img + ((size_t)ch * H + r0 + r) * W + 4 * c4);
                *reinterpret_cast<float4 *>(sv + ch * SVC + r * W + 4 * c4) = val;
            }
            const int X4 = (W + halo) / 4, H4 = halo / 4;      // the first H4 pieces of a row are the halo
            for (int idx = tid; idx < C * xrows * X4; idx += 256) {
                const int c4 = idx % X4, rr = idx / X4;
                const int ch = rr / xrows, r = rr - ch * xrows;
                const int gr = r0 - (k - 1) + r;
                float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
                if (gr >= 0 && c4 >= H4)
                    val = *reinterpret_cast<const float4 *>(x + img + ((size_t)ch * H + gr) * W + 4 * (c4 - H4));
                *reinterpret_cast<float4 *>(sx + ch * SXC + r * XW + 4 * c4) = val;
            }
        } else {
            for (int idx = tid; idx < Cv * rows * W; idx += 256) {
                const int c = idx % W, r = (idx / W) % rows, ch = idx / (W * rows);
                sv[ch * SVC + r * W + c] = v[img + ((size_t)ch * H + r0 + r) * W + c];
            }
            const int xcols = W + halo;
            for (int idx = tid; idx < C * xrows * xcols; idx += 256) {
                const int cc = idx % xcols, rr = (idx / xcols) % xrows, ch = idx / (xcols * xrows);
                const int gr = r0 - (k - 1) + rr, gc = cc - halo;
                sx[ch * SXC + rr * XW + cc] =
                    (gr >= 0 && gc >= 0) ? x[img + ((size_t)ch * H + gr) * W + gc] : 0.0f;
            }
        }
        __syncthreads();
        if (vec == 2 && it + 1 < trips) {
            // the next chunk (or the next image's only chunk) travels while the matrix cores work on this one
            const int rn = ipw > 1 ? 0 : r0 + RT;
            const size_t img_n = ipw > 1 ? img + img_stride : img;
#pragma unroll
            for (int i = 0; i < kDwPre; ++i) {
                const bool in = p_r[i] >= 0 && rn + p_r[i] < H;
                const size_t go = img_n + (p_r[i] >= 0 ? p_go[i] : 0) + (size_t)(in ? rn : 0) * W;
                // (a piece whose channel is missing in one of the blocks reads the block's first channel: unused)
                const float4 a4 = *reinterpret_cast<const float4 *>(v + (p_hv[i] ? go : img_n));
                const float4 b4 = *reinterpret_cast<const float4 *>(x + (p_hx[i] ? go : img_n));
                pv[i] = a4;
                px[i] = in ? b4 : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }

        if (vec) {
            // W is a multiple of 4: a wave takes whole rows, four pixels (lanes kk = 0..3) per instruction and
            // kDwUnroll such quads per trip, so that the tile offsets inside a trip are immediates
            const int WQ = W >> 2, NBLK = WQ / kDwUnroll;
            // wide rows: the four waves share every row (blocks wave, wave+4, ...); narrow rows: a wave
            // takes whole rows
            const bool share = NBLK >= 4;
            const int pr_step = share ? 1 : 4, q_first = share ? wave : 0, q_step = share ? 4 : 1;
            for (int pr = share ? 0 : wave; pr < rows; pr += pr_step) {
                const float *ap = sv + aoff + pr * W + kk;
                const float *bp = sx + pr * XW + kk;
                for (int blk = q_first; blk < NBLK; blk += q_step) {
                    const int qc = blk * kDwUnroll;
                    float av[kDwUnroll];
#pragma unroll
                    for (int u = 0; u < kDwUnroll; ++u)
                        av[u] = ap[4 * (qc + u)];
#pragma unroll
                    for (int s = 0; s < NS; ++s) {
                        const float *bs = bp + boff[s] + 4 * qc;
#pragma unroll
                        for (int u = 0; u < kDwUnroll; ++u)
                            acc[s] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u], bs[4 * u], acc[s], 0, 0, 0);
                    }
                }
                for (int qc = NBLK * kDwUnroll + q_first; qc < WQ; qc += q_step) {
                    const float av = ap[4 * qc];
#pragma unroll
                    for (int s = 0; s < NS; ++s)
                        acc[s] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bp[boff[s] + 4 * qc], acc[s], 0, 0, 0);
                }
            }
        } else {
            const int npix = rows * W;
            const int ngroups = (npix + 3) / 4;
            for (int q = wave; q < ngroups; q += 4) {
                const int p = 4 * q + kk;
                const bool pv = p < npix;
                const int pr = pv ? p / W : 0, pc = pv ? p - pr * W : 0;
                const float avl = sv[aoff + pr * W + pc];
                const float av = pv ? avl : 0.0f;       // pixels past the end contribute nothing
                const float *bp = sx + pr * XW + pc;
#pragma unroll
                for (int s = 0; s < NS; ++s)
                    acc[s] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bp[boff[s]], acc[s], 0, 0, 0);
            }
        }
        if (ipw > 1)
            img += img_stride;
    }
    __syncthreads();        // tiles no longer needed
    // lane (nn, g = kk) register (s, j) holds entry (o = 4g + j, col = 16s + nn)
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            sred[tid * (NS * 4) + s * 4 + j] = acc[s][j];
    __syncthreads();
    for (int e = tid; e < P; e += 256) {
        const int o = e / NCOL, col = e % NCOL;
        const int s = col >> 4, cn = col & 15, g = o >> 2, j = o & 3;
        float sum = 0.0f;
        for (int wv = 0; wv < 4; ++wv)
            sum += sred[(wv * 64 + g * 16 + cn) * (NS * 4) + s * 4 + j];
        part[(size_t)blockIdx.x * (pstride ? pstride : P) + e] = sum;
    }
}

constexpr int kDwChannelBlock = 16;
constexpr int kDwMaxNs = 10;        // accumulators (blocks of 16 columns) a wave holds

// Input channels of one block of the result: their Cx k k "shifted x" columns have to fit the accumulators
// (16 channels up to k = 3, 6 at k = 5), and a block has at most 16 of them.
static int dw_x_block(int C, int k)
{
    int cx = (16 * kDwMaxNs) / (k * k);
    cx = cx > kDwChannelBlock ? kDwChannelBlock : cx;
    return cx > C ? C : cx;
}

// one GEMM up to 16 channels when the columns fit; otherwise blocks of (at most 16 output) x (dw_x_block input)
// channels, all blocks in one launch
bool dw_mfma_supported(int C, int k)
{
    return C >= 1 && C <= 64 && k >= 1 && dw_x_block(C, k) >= 1;
}

// Row chunking of pass 1 for one block of Cv output x Cx input channels: tiles (or the reduction buffer that reuses
// them) must fit the LDS budget.  p.nparts = B * G partial rows per block, G workgroups per image each looping over chunks.
static DwPlan plan_dw_mfma_block(int B, int Cv, int C, int H, int W, int k, int nblocks = 1)
{
    DwPlan p{};
    const int CM = Cv > C ? Cv : C;
    const size_t P = (size_t)Cv * C * k * k;
    const size_t NS = ((size_t)C * k * k + 15) / 16;
    const size_t red = 256 * NS * 4;
    // strides: v rows stay contiguous, its channel stride is 4 (mod 64) so that the 16 output channels of
    // an A operand read fall into different banks; the x tile's row and channel pads are searched
    auto svc_for = [&](int rt) {
        const int base = rt * W;
        return base + ((4 - base % 64) + 64) % 64;
    };
    auto lds_with = [&](int rt, int xw, int sxc) {
        const size_t tiles = (size_t)CM * svc_for(rt) + (size_t)C * sxc;
        return sizeof(float) * (tiles > red ? tiles : red);
    };
    const int halo = dw_halo(k);
    auto lds_for = [&](int rt) { return lds_with(rt, W + halo, (rt + k - 1) * (W + halo)); };
    // Rows of 16-byte pieces take the streaming mode (if the pointers are aligned too): registers limit it
    // to two workgroups per compute unit, so its tiles may be larger, as long as a thread's share of a
    // tile still fits its kDwPre registers.
    const bool stream_shape = (W % 4) == 0;
    const size_t budget = stream_shape ? kDwStreamLdsBudget : kDwLdsBudget;
    if (lds_for(1) > budget)
        return p;
    // chunks of 8 rows; kernels of more than 9 rows take 16, so that a chunk still covers the k - 1 halo rows the
    // streaming mode carries over from the chunk before, and so do images of at most 16 rows, which are then one
    // chunk and can go several to a workgroup - where that still leaves a workgroup per compute unit
    // (the blocks of a blocked result that share a launch count as images here)
    const int shared = nblocks < kChainMaxLayers ? nblocks : kChainMaxLayers;
    const bool tall_chunks = stream_shape && (k - 1 > 8 || H <= 16) && (long)B * shared * ((H + 15) / 16) >= 320;
    const int rt_max = tall_chunks ? 16 : 8;
    int rt = H < rt_max ? H : rt_max;
    while (rt > 1 && (lds_for(rt) > budget || (stream_shape && rt > k - 1 && CM * rt * (W / 4) > 256 * kDwPre)))
        --rt;
    p.rt = rt;
    p.nchunks = (H + rt - 1) / rt;
    p.svc = svc_for(rt);
    p.xw = W + halo;
    p.sxc = (rt + k - 1) * p.xw;
    {
        // bank conflicts of the B operand reads: lane (nn, kk) of instruction s reads
        // i*sxc + a*xw + b + kk for column 16s + nn = (i, a, b); cost = cycles the read takes in the model below.
        // The search costs a fraction of a millisecond of host time, so the last few answers are remembered
        // per thread (a call may plan several kernel sizes of one shape).
        struct Memo { int C, k, rt, W, xw, sxc; };
        constexpr int kMemos = 16;
        static thread_local Memo memos[kMemos] = {};
        static thread_local int memo_next = 0;
        Memo *hit = nullptr;
        for (int m = 0; m < kMemos; ++m)
            if (memos[m].C == 100 * Cv + C && memos[m].k == k && memos[m].rt == rt && memos[m].W == W)
                hit = &memos[m];
        Memo memo = hit ? *hit : Memo{0, 0, 0, 0, 0, 0};
        if (!hit) {
            const int ncol = C * k * k;
            // LDS model (measured with strided 4-byte reads: stride 32 words costs as much as stride 64, and
            // moving the upper 32 lanes by 64 words costs nothing): 32 banks of 4 bytes, a 64-lane read is
            // served as two halves of 32 lanes, a half takes as many cycles as its fullest bank has distinct
            // addresses.
            auto cost = [&](int xw, int sxc) {
                int total = 0;
                for (int s = 0; s < (int)NS; ++s)
                    for (int half = 0; half < 2; ++half) {
                        int addr[32], per_bank[32] = {0};
                        for (int h = 0; h < 32; ++h) {
                            const int l = 32 * half + h, nn = l & 15, kk = l >> 4;
                            const int col = 16 * s + nn < ncol ? 16 * s + nn : 0;
                            addr[h] = (col / (k * k)) * sxc + ((col / k) % k) * xw + col % k + kk;
                            bool seen = false;
                            for (int m = 0; m < h; ++m)
                                seen = seen || addr[m] == addr[h];
                            if (!seen)
                                ++per_bank[addr[h] % 32];
                        }
                        int worst = 1;
                        for (int bank = 0; bank < 32; ++bank)
                            worst = per_bank[bank] > worst ? per_bank[bank] : worst;
                        total += worst;
                    }
                return total;
            };
            Memo m = {100 * Cv + C, k, rt, W, p.xw, p.sxc};
            int best = cost(p.xw, p.sxc);
            for (int rp = 0; rp <= 12; rp += 4)
                for (int cp = 0; cp <= 60; cp += 4) {
                    const int xw = W + halo + rp, sxc = (rt + k - 1) * xw + cp;
                    if (lds_with(rt, xw, sxc) > budget)             // same number of workgroups per CU as unpadded
                        continue;
                    const int c = cost(xw, sxc);
                    if (c < best) {
                        best = c;
                        m.xw = xw;
                        m.sxc = sxc;
                    }
                }
            memo = m;
            memos[memo_next] = m;
            memo_next = (memo_next + 1) % kMemos;
        }
        p.xw = memo.xw;
        p.sxc = memo.sxc;
    }
    // Workgroups per image: a workgroup streams through a contiguous range of chunks and re-reads only the
    // k-1 halo rows at the start of its range, so few long ranges are better than many short ones, as long
    // as every compute unit gets a workgroup or two per layer.
    int g = (320 + B * shared - 1) / (B * shared);
    if (g > p.nchunks) g = p.nchunks;
    if (g < 1) g = 1;
    g = (p.nchunks + (p.nchunks + g - 1) / g - 1) / ((p.nchunks + g - 1) / g);      // no empty workgroups
    p.groups = g;
    // images of a single chunk in large batches: a workgroup takes several, as long as one and a half workgroups
    // per compute unit are left - or three quarters of one for the blocks of a blocked result, whose rows of
    // partial sums are long (measured at 48, 32, 24 and 12 channels on 8 x 8 images, 100 to 4096 of them)
    p.ipw = 1;
    if (p.nchunks == 1) {
        const long ipw = (long)B * shared / (nblocks > 1 ? 192 : 384);
        p.ipw = ipw > 16 ? 16 : (ipw > 1 ? (int)ipw : 1);
    }
    p.nparts = (size_t)((B + p.ipw - 1) / p.ipw) * g;
    p.lds = lds_with(rt, p.xw, p.sxc);
    p.bytes = ((p.nparts * P * sizeof(float)) + 255) / 256 * 256;
    return p;
}

DwPlan plan_dw_mfma(int B, int C, int H, int W, int k)
{
    if (!dw_mfma_supported(C, k))
        return DwPlan{};
    const int cbv = C < kDwChannelBlock ? C : kDwChannelBlock, cbx = dw_x_block(C, k);
    if (cbv == C && cbx == C)
        return plan_dw_mfma_block(B, C, C, H, W, k);        // one GEMM
    // blocks of cbv output x cbx input channels: the plan of one block; up to kChainMaxLayers blocks share a
    // launch, each with its own partial rows
    const size_t nblocks = (size_t)((C + cbv - 1) / cbv) * ((C + cbx - 1) / cbx);
    DwPlan p = plan_dw_mfma_block(B, cbv, cbx, H, W, k, (int)nblocks);
    p.cb = p.rt ? cbv : 0;
    p.cbx = cbx;
    p.bytes *= nblocks < (size_t)kChainMaxLayers ? nblocks : (size_t)kChainMaxLayers;
    return p;
}

// The same plan for one launch over `layers` layers: fewer, longer chunk ranges per image, about two
// workgroups per compute unit in all (a workgroup's set-up and its final reduction cost about as much as
// two chunks).  Never more partial rows than plan_dw_mfma's, so the same workspace serves.
DwPlan plan_dw_mfma_layers(int layers, int B, int C, int H, int W, int k)
{
    DwPlan p = plan_dw_mfma(B, C, H, W, k);
    if (!p.rt || layers <= 1)
        return p;
    const long per_round = 512;
    int g = (int)((per_round + (long)B * layers - 1) / ((long)B * layers));
    if (g > p.groups) g = p.groups;
    if (g < 1) g = 1;
    g = (p.nchunks + (p.nchunks + g - 1) / g - 1) / ((p.nchunks + g - 1) / g);      // no empty workgroups
    p.groups = g;
    const int ipw = p.ipw > 1 ? p.ipw : 1;
    p.nparts = (size_t)((B + ipw - 1) / ipw) * g;
    return p;
}

// C = x channels of the block (= all channels without blocking), Cv = v channels, Ctot = channels of the tensors
template <int NS>
static bool launch_ns(const DwBatch &batch, int layers, float *part, const DwPlan &p, int B, int C, int H, int W,
                      int k, hipStream_t stream, int Cv, int Ctot, int pstride)
{
    // 16-byte tile loads need rows that start on 16-byte boundaries
    int vec = (W % 4) == 0;
    for (int l = 0; l < layers; ++l)
        if (((size_t)batch.x[l] | (size_t)batch.v[l]) & 15)
            vec = 0;
    // streaming mode: the halo rows come from one chunk before, and a thread's share of a tile fits its registers
    if (vec && p.rt >= k - 1 && (C > Cv ? C : Cv) * p.rt * (W / 4) <= 256 * kDwPre)
        vec = 2;
    if (!ensure_dynamic_lds(reinterpret_cast<const void *>(&k_dw_partial_mfma<NS>), p.lds))
        return false;
    const int ipw = p.ipw > 1 ? p.ipw : 1;
    hipLaunchKernelGGL(k_dw_partial_mfma<NS>, dim3((unsigned)(p.nparts * layers)), dim3(256), p.lds, stream, batch,
                       part, (B + ipw - 1) / ipw, C, H, W, k, p.rt, p.nchunks, p.groups, vec, p.xw, p.sxc, p.svc, Cv,
                       Ctot, pstride, ipw, B);
    return true;
}

// Pass 1 for `layers` independent (x, v) pairs in one launch; part holds layers * p.nparts rows.
static int launch_dw_partial_batch(const DwBatch &batch, int layers, float *part, const DwPlan &p, int B, int C,
                                   int H, int W, int k, hipStream_t stream, int Cv = 0, int Ctot = 0,
                                   int pstride = 0)
{
    Cv = Cv ? Cv : C;
    Ctot = Ctot ? Ctot : C;
    const int ns = (C * k * k + 15) / 16;
    bool ok = false;
    switch (ns) {
    case 1: ok = launch_ns<1>(batch, layers, part, p, B, C, H, W, k, stream, Cv, Ctot, pstride); break;
    case 2: ok = launch_ns<2>(batch, layers, part, p, B, C, H, W, k, stream, Cv, Ctot, pstride); break;
    case 3: ok = launch_ns<3>(batch, layers, part, p, B, C, H, W, k, stream, Cv, Ctot, pstride); break;
    case 4: ok = launch_ns<4>(batch, layers, part, p, B, C, H, W, k, stream, Cv, Ctot, pstride); break;
    case 5: ok = launch_ns<5>(batch, layers, part, p, B, C, H, W, k, stream, Cv, Ctot, pstride); break;
    case 6: ok = launch_ns<6>(batch, layers, part, p, B, C, H, W, k, stream, Cv, Ctot, pstride); break;
    case 7: ok = launch_ns<7>(batch, layers, part, p, B, C, H, W, k, stream, Cv, Ctot, pstride); break;
    case 8: ok = launch_ns<8>(batch, layers, part, p, B, C, H, W, k, stream, Cv, Ctot, pstride); break;
    case 9: ok = launch_ns<9>(batch, layers, part, p, B, C, H, W, k, stream, Cv, Ctot, pstride); break;
    case 10: ok = launch_ns<10>(batch, layers, part, p, B, C, H, W, k, stream, Cv, Ctot, pstride); break;
    default: return INVCONV_ERR_UNSUPPORTED;
    }
    if (!ok)
        return INVCONV_ERR_UNSUPPORTED;
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

int launch_dw_mfma(const float *x, const float *v, float *dw, float *part, const DwPlan &p, int B, int C, int H,
                   int W, int k, hipStream_t stream, float sign, bool masked)
{
    if (!masked && !p.cb)
        return INVCONV_ERR_VARIANT;     // (one block: pass 1 alone gives the unmasked rows)
    DwBatch batch{};
    if (p.cb) {
        // More than 16 channels: the result is cut into blocks of at most 16 output x 16 input channels.  All
        // blocks (at most 16: C <= 64) are the "layers" of ONE first pass and ONE second pass; a launch pair
        // per block made the weight gradient of 48 x 8 x 8 images eighteen launches of a few microseconds.
        const size_t plane = (size_t)H * W;
        DwBlocks blocks{};
        const int pstride = p.cb * p.cbx * k * k;
        auto flush = [&]() -> int {
            if (!blocks.n)
                return INVCONV_OK;
            if (int s = launch_dw_partial_batch(batch, blocks.n, part, p, B, p.cbx, H, W, k, stream, p.cb, C, pstride))
                return s;
            if (int s = launch_dw_reduce_blocks(part, (int)p.nparts, dw, blocks, C, k, pstride, stream, sign, masked))
                return s;
            blocks.n = 0;       // (launches of one stream run in order: the next group may reuse the partial rows)
            return INVCONV_OK;
        };
        for (int o0 = 0; o0 < C; o0 += p.cb)
            for (int i0 = 0; i0 < C; i0 += p.cbx) {
                const int Cv = C - o0 < p.cb ? C - o0 : p.cb, Cx = C - i0 < p.cbx ? C - i0 : p.cbx;
                const int l = blocks.n++;
                batch.x[l] = x + i0 * plane;
                batch.v[l] = v + o0 * plane;
                batch.cx[l] = blocks.cx[l] = (unsigned char)Cx;
                batch.cv[l] = blocks.cv[l] = (unsigned char)Cv;
                blocks.o0[l] = (unsigned char)o0;
                blocks.i0[l] = (unsigned char)i0;
                if (blocks.n == kChainMaxLayers)
                    if (int s = flush())
                        return s;
            }
        return flush();
    }
    batch.x[0] = x;
    batch.v[0] = v;
    if (int s = launch_dw_partial_batch(batch, 1, part, p, B, C, H, W, k, stream))
        return s;
    return launch_dw_reduce(part, (int)p.nparts, dw, C, k, stream, sign);
}

// Pass 1 alone: p.nparts rows of C*C*k*k un-negated, unmasked partial sums in `part`
int launch_dw_mfma_partial(const float *x, const float *v, float *part, const DwPlan &p, int B, int C, int H, int W,
                           int k, hipStream_t stream)
{
    DwBatch batch{};
    batch.x[0] = x;
    batch.v[0] = v;
    return launch_dw_partial_batch(batch, 1, part, p, B, C, H, W, k, stream);
}

// dL/dw of `layers` layers: one pass-1 launch over all of them, then one pass 2 per layer.
// part must hold layers * p.bytes bytes.
int launch_dw_mfma_layers(const float *const *x, const float *const *v, float *const *dw, int layers, float *part,
                          const DwPlan &p, int B, int C, int H, int W, int k, hipStream_t stream)
{
    if (layers < 1 || layers > kChainMaxLayers)
        return INVCONV_ERR_SHAPE;
    DwBatch batch{};
    for (int l = 0; l < layers; ++l) {
        batch.x[l] = x[l];
        batch.v[l] = v[l];
    }
    if (int s = launch_dw_partial_batch(batch, layers, part, p, B, C, H, W, k, stream))
        return s;
    return launch_dw_reduce_layers(part, (int)p.nparts, dw, layers, C, k, stream);
}

}  // namespace invconv
