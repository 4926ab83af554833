// Wavefront solve for many channels (C = 17 .. 48, laid out for multiples of 4; k = 3): the shapes a flow reaches
// after two squeezes (Section 4.1).  gfx950 only.
//
// With folded weights (Linv = inverse of the current-pixel block, Cf_tap = Linv W_tap) the channels of a pixel
// are independent:  x_p = Linv y_p - sum_{tap} Cf_tap x_{p - tap}  (Eq. 1 rearranged), and at this channel
// count the per-tap mixing is a real contraction: for the 16 pixels that a band of 16 rows has on one
// anti-diagonal it is a [16 out] x [C in] x [16 pixels] product per tap and block of 16 output channels, i.e.
// C/4 v_mfma_f32_16x16x4_f32 whose A operand is a weight tile and whose B operand is the history of x.
//
// One workgroup per image; wave (band, ob) owns rows 16 band .. 16 band + 15 and output channels 16 ob ..
// 16 ob + 15.  All rows run in lock step: at step t row r is at column t - r, so pixel (r - da, c - db) was
// finished da + db steps ago by the wave that owns row r - da.  The results of the last 2k - 1 steps live in
// an LDS ring, ring[t mod 5][row + k - 1][channel] (k - 1 rows of zeros on top, zeros for pixels outside the
// image), so a tap's B operand is one LDS read per lane and no message travels between waves.  The folded
// weights live in LDS as well, [tap][out][in], rows padded to an odd stride so that the 16 rows of a tile
// fall into different banks.  One workgroup barrier per step: a wave writes slot t mod 5 only after every
// wave has finished reading for step t - 1, and step t reads slots t - 1 .. t - 4.
// The transposed solve is the same kernel in mirrored coordinates (DIR = 1).
#include "invconv_common.h"
#include "invconv_launch.h"
#include "invconv_tri_inverse.h"
#include <type_traits>

namespace invconv {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWideK = 3;
constexpr int kWideRing = 2 * kWideK - 1;

__host__ __device__ constexpr int wide_out_blocks(int C) { return (C + 15) / 16; }

// Weight preparation of a workgroup: sWt[tap][out (padded to whole blocks of 16)][in, row stride C + 1] = Linv for
// tap 0 and -Linv W_tap for the others, from oriented, masked kernel entries read straight from global memory.
// The eight products Linv W_tap (C^3 multiply-adds each) run on the matrix cores, four taps at a time: a task is
// one 16 x 16 block of one product, the waves take tasks round robin, and since Linv is lower triangular a
// block of rows 16 ob .. needs only the first 4 (ob + 1) of the C/4 instructions.  Operands come from LDS with
// one 4-byte read each: Linv[o][j] with an odd row stride (the 16 rows of an A read in different banks) and
// W_tap[j][i] with a row stride of 48 (the two k-slots of a half-wave 16 banks apart).
// scratch: wide_fold_scratch_floats(C) floats.  Ends with a barrier.
constexpr int kWideTapStride = 48;      // row stride of the staged taps: C <= 48, and 48 mod 32 = 16
__host__ __device__ constexpr size_t wide_fold_scratch_floats(int C)
{
    return (size_t)C * C + (size_t)16 * wide_out_blocks(C) * (C + 1) + (size_t)4 * C * kWideTapStride +
           tri_inverse_tmp_floats();
}

// Cr: the channels the image really has (4 CQ - 3 .. 4 CQ); the surplus ones are given an identity current-pixel
// block and no other taps, so they solve to their (zero) input and touch nothing else.
template <int CQ, int DIR, bool PAD>
__device__ __forceinline__ void wide_fold_weights(const float *__restrict__ w, float *sWt, float *scratch, int Cr_arg)
{
    constexpr int C = 4 * CQ, K = kWideK, NT = K * K;
    const int Cr = PAD ? Cr_arg : C;
    constexpr int OB = wide_out_blocks(C), OR = 16 * OB, CPAD = C + 1;
    constexpr int LP = C + 1, TP = kWideTapStride;
    static_assert(C <= TP && OR <= TP && NT == 9, "tap staging is laid out for at most 48 channels, 3 x 3 taps");
    float *sL = scratch, *sLinv = sL + C * C, *sTap = sLinv + OR * LP;       // [C][C], [OR][LP], [4][C][TP], inverse's
    const int tid = threadIdx.x, nt = blockDim.x;
    auto entry = [&](int tp, int o, int i) -> float {
        const int a = K - 1 - tp / K, b = K - 1 - tp % K;
        const bool real = o < Cr && i < Cr;
        const int oc = real ? o : 0, ic = real ? i : 0;
        const int oo = DIR ? Cr - 1 - ic : oc, ii = DIR ? Cr - 1 - oc : ic;
        const float v = w[((oo * Cr + ii) * K + a) * K + b];
        if (!real)
            return (tp == 0 && o == i) ? 1.0f : 0.0f;
        return (tp == 0 && ii > oo) ? 0.0f : v;
    };
    // four taps into LDS, sixteen loads of a thread in flight; columns C .. TP-1 and the rows of Linv past C are
    // zeros (they feed padding rows and columns of the blocks)
    auto stage = [&](int tp0) {
        for (int base = tid; base < 4 * C * C; base += 16 * nt) {
            float v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int idx = base + u * nt;
                const int q = idx / (C * C), e = idx % (C * C);
                v[u] = idx < 4 * C * C ? entry(tp0 + q, e / C, e % C) : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int idx = base + u * nt;
                const int q = idx / (C * C), e = idx % (C * C);
                if (idx < 4 * C * C)
                    sTap[(q * C + e / C) * TP + e % C] = v[u];
            }
        }
    };
    for (int idx = tid; idx < C * C; idx += nt)
        sL[idx] = entry(0, idx / C, idx % C);
    if constexpr (C < TP) {
        for (int idx = tid; idx < 4 * C * (TP - C); idx += nt)
            sTap[(idx / (TP - C)) * TP + C + idx % (TP - C)] = 0.0f;
    }
    for (int idx = tid; idx < (OR - C) * LP; idx += nt)
        sLinv[C * LP + idx] = 0.0f;
    stage(1);
    __syncthreads();
    // Inverse of the lower-triangular block in 16 x 16 blocks by the whole workgroup (one thread per column, the
    // column in registers, was a chain of C dependent rows: 8 us of one wave at 48 channels)
    tri_inverse_blocks<C>(sL, sLinv, LP, sTap + 4 * C * TP);
    for (int it = tid; it < OR * C; it += nt) {
        const int o = it / C, i = it % C;
        sWt[o * CPAD + i] = sLinv[o * LP + i];      // tap 0 (rows past C: zeros)
    }
    const int wave = tid >> 6, lane = tid & 63, nwv = nt >> 6, n = lane & 15, g = lane >> 4;
    // taps 5 .. 8 travel from memory while the matrix cores work on taps 1 .. 4 (a workgroup has at least OB waves)
    constexpr int NPRE = (4 * C * C + 64 * OB - 1) / (64 * OB);
    float pre[NPRE];
#pragma unroll
    for (int u = 0; u < NPRE; ++u) {
        const int idx = tid + u * nt;
        const int q = idx / (C * C), e = idx % (C * C);
        pre[u] = idx < 4 * C * C ? entry(5 + q, e / C, e % C) : 0.0f;
    }
    for (int half = 0; half < 2; ++half) {
        if (half) {
#pragma unroll
            for (int u = 0; u < NPRE; ++u) {
                const int idx = tid + u * nt;
                const int q = idx / (C * C), e = idx % (C * C);
                if (idx < 4 * C * C)
                    sTap[(q * C + e / C) * TP + e % C] = pre[u];
            }
            __syncthreads();
        }
        for (int task = wave; task < 4 * OB * OB; task += nwv) {
            const int q = task / (OB * OB), ob = (task / OB) % OB, ib = task % OB;
            const float *ap = sLinv + (16 * ob + n) * LP + g;           // A[m = n][k = g] = Linv[16 ob + n][4 c + g]
            const float *bp = sTap + (q * C + g) * TP + 16 * ib + n;    // B[k = g][n] = W[4 c + g][16 ib + n]
            const int nc = 4 * (ob + 1) < CQ ? 4 * (ob + 1) : CQ;
            f32x4 acc0 = f32x4{0.f, 0.f, 0.f, 0.f}, acc1 = f32x4{0.f, 0.f, 0.f, 0.f};
            // four instructions' operands are read together, ahead of the instructions (past nc: a valid address,
            // a zero B operand)
            for (int c = 0; c < nc; c += 4) {
                float a[4], b[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int cc = c + u < nc ? c + u : nc - 1;
                    a[u] = ap[4 * cc];
                    const float bv = bp[4 * cc * TP];
                    b[u] = c + u < nc ? bv : 0.0f;
                }
                acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[0], b[0], acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[1], b[1], acc1, 0, 0, 0);
                acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[2], b[2], acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[3], b[3], acc1, 0, 0, 0);
            }
            const f32x4 acc = acc0 + acc1;
            // D[m = 4 g + j][n]: rows 16 ob + 4 g + j, column 16 ib + n
            if (16 * ib + n < C) {
                float *dst = sWt + ((1 + 4 * half + q) * OR + 16 * ob + 4 * g) * CPAD + 16 * ib + n;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    dst[j * CPAD] = -acc[j];
            }
        }
        __syncthreads();
    }
}

// PAD: the image has Cr < 4 CQ channels (otherwise Cr is the compile-time constant 4 CQ: the clamps and
// predicates on the channel index fold away, which is worth 5-13 % at 32 and 48 channels)
template <int CQ, int DIR, bool PAD>
__global__ __launch_bounds__(1024) void k_solve_wide(const float *__restrict__ in, const float *__restrict__ w,
                                                    float *__restrict__ out, int H, int W, int NB, float *logdet,
                                                    int Cr_arg)
{
    constexpr int C = 4 * CQ, K = kWideK, NT = K * K, R = kWideRing;
    const int Cr = PAD ? Cr_arg : C;
    constexpr int OB = wide_out_blocks(C), OR = 16 * OB, CPAD = C + 1;
    extern __shared__ float smem[];
    const int HP = 16 * NB + K - 1;
    float *sWt = smem;                          // [NT][OR][CPAD]: tap 0 = Linv, the others = -Linv W_tap
    float *ring = sWt + NT * OR * CPAD;         // [R][HP][CPAD]
    // (the ring's memory is the folding scratch first)
    const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int band = wave / OB, ob = wave % OB;
    const int n = lane & 15, g = lane >> 4;

    wide_fold_weights<CQ, DIR, PAD>(w, sWt, ring, Cr);
    for (int idx = tid; idx < R * HP * CPAD; idx += nt)
        ring[idx] = 0.0f;
    __syncthreads();

    // ---- this lane: pixel row r (B operand column n), input channels 4 c4 + g (K slot g),
    //      A operand row m = n -> output channel 16 ob + n; results: output channels 16 ob + 4 g + j
    const int r = 16 * band + n;
    const bool row_ok = r < H;
    const size_t img = (size_t)blockIdx.x * Cr * H * W;
    const int a_base = (16 * ob + n) * CPAD + g;                 // + tp * OR * CPAD + 4 c4
    const int b_row = (r + K - 1) * CPAD + g;                    // + slot * HP * CPAD - da * CPAD + 4 c4
    const int o_first = 16 * ob + 4 * g;                         // first of this lane's four output channels
    auto gaddr = [&](int ch, int rr, int cc) -> size_t {     // ch < Cr
        return img + ((size_t)(DIR ? Cr - 1 - ch : ch) * H + (DIR ? H - 1 - rr : rr)) * W + (DIR ? W - 1 - cc : cc);
    };
    auto load_y = [&](int t, float (&yv)[CQ]) {
        const int c = t - r;
        const bool ok = row_ok && (unsigned)c < (unsigned)W;
        const int rr = row_ok ? r : 0, cc = ok ? c : 0;
#pragma unroll
        for (int c4 = 0; c4 < CQ; ++c4) {
            const int ch = 4 * c4 + g;
            const float v = in[gaddr(ch < Cr ? ch : 0, rr, cc)];
            yv[c4] = (ok && ch < Cr) ? v : 0.0f;
        }
    };
    float ycur[CQ], ynext[CQ];
    load_y(0, ycur);
    const int nsteps = H + W - 1;
    int tm = 0;                                                 // t mod R
    for (int t = 0; t < nsteps; ++t) {
        load_y(t + 1, ynext);                                   // one step ahead (past the last step: zeros)
        // Operands of tap tp + 1 are read from LDS while the matrix cores work on tap tp (two register
        // sets), and the products alternate between two accumulators: neither the LDS latency nor the
        // latency of a dependent matrix instruction lies on every instruction's path.
        float opa[2][CQ], opb[2][CQ];
        auto read_tap = [&](int tp, float (&oa)[CQ], float (&ob_)[CQ]) {
            const int da = tp / K, db = tp % K, lag = da + db;
            int slot = tm - lag;
            slot += slot < 0 ? R : 0;
            const float *bp = ring + slot * HP * CPAD + b_row - da * CPAD;
            const float *ap = sWt + tp * OR * CPAD + a_base;
#pragma unroll
            for (int c4 = 0; c4 < CQ; ++c4) {
                oa[c4] = ap[4 * c4];
                ob_[c4] = tp == 0 ? ycur[c4] : bp[4 * c4];
            }
        };
        f32x4 acc0 = f32x4{0.f, 0.f, 0.f, 0.f}, acc1 = f32x4{0.f, 0.f, 0.f, 0.f};
        read_tap(0, opa[0], opb[0]);
#pragma unroll
        for (int tp = 0; tp < NT; ++tp) {
            if (tp + 1 < NT)
                read_tap(tp + 1, opa[(tp + 1) & 1], opb[(tp + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);      // keep the reads above ahead of the products below
#pragma unroll
            for (int c4 = 0; c4 < CQ; ++c4) {
                if (c4 & 1)
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(opa[tp & 1][c4], opb[tp & 1][c4], acc1, 0, 0, 0);
                else
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(opa[tp & 1][c4], opb[tp & 1][c4], acc0, 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        const f32x4 acc = acc0 + acc1;
        // The next step's input is taken over BEFORE this step's global stores are issued: vector memory
        // operations complete in order, so waiting for the loads behind the stores would wait for the stores'
        // round trip in every step.
#pragma unroll
        for (int c4 = 0; c4 < CQ; ++c4) {
            ycur[c4] = ynext[c4];
            asm volatile("" : "+v"(ycur[c4]));
        }
        __builtin_amdgcn_sched_barrier(0);
        const int c = t - r;
        const bool ok = row_ok && (unsigned)c < (unsigned)W;
        float *rp = ring + tm * HP * CPAD + (r + K - 1) * CPAD + o_first;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (o_first + j < C) {
                rp[j] = ok ? acc[j] : 0.0f;                     // pixels outside the image count as zeros
                if (ok && o_first + j < Cr)
                    out[gaddr(o_first + j, r, c)] = acc[j];
            }
        }
        tm = tm + 1 == R ? 0 : tm + 1;
        // workgroup barrier that orders LDS only: this step's global stores stay in flight across it (a full
        // __syncthreads() would wait for them at every step)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    }
    if (logdet && blockIdx.x == 0 && wave == 0)
        wave_logdet_any(w, Cr, K, H, W, logdet);
}

// ---------------------------------------------------------------------------
// The same solve for workgroups of at most twelve waves (e.g. 48 channels on 32 rows: 2 bands x 3 blocks of
// output channels), where a wave may hold its whole weight tile - 9 taps x C/4 A operands - in registers:
//   * no weight is read from LDS inside the step loop (it was half of the LDS traffic);
//   * the rings keep a pixel's channels permuted, channel 4 c4 + g at position g C/4 + c4, so that the C/4
//     B operands of lane (n, g) are contiguous and come in with 16-byte (8-byte) LDS reads;
//   * the input y takes the same route as x: the wave of output block ob fetches only channels 16 ob ..
//     16 ob + 15 of its rows' pixels of the next step (four 4-byte loads per lane instead of C/4 - the
//     address unit handles one lane per clock, and every wave of a band used to fetch all C channels) and
//     puts them into a two-slot LDS buffer, from which all waves of the band take the B operand of Linv y.
// Same arithmetic in the same order as k_solve_wide.  The LDS first holds the folded weights, then the rings.
// ---------------------------------------------------------------------------
template <int CQ>
__host__ __device__ constexpr int wide_vec() { return CQ % 4 == 0 ? 4 : (CQ % 2 == 0 ? 2 : 1); }

template <int CQ>
__device__ __forceinline__ void wide_read_operands(const float *p, float (&o)[CQ])
{
    constexpr int VW = wide_vec<CQ>();
    if constexpr (VW == 4) {
#pragma unroll
        for (int i = 0; i < CQ / 4; ++i) {
            const f32x4 v = *reinterpret_cast<const f32x4 *>(p + 4 * i);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                o[4 * i + j] = v[j];
        }
    } else if constexpr (VW == 2) {
#pragma unroll
        for (int i = 0; i < CQ / 2; ++i) {
            const float2 v = *reinterpret_cast<const float2 *>(p + 2 * i);
            o[2 * i] = v.x;
            o[2 * i + 1] = v.y;
        }
    } else {
#pragma unroll
        for (int i = 0; i < CQ; ++i)
            o[i] = p[i];
    }
}

// Issue order of one tap (CQ matrix products and the LDS reads of the next tap's operands): a product, a read, a
// product, a read, ... A wave issues in order and a product occupies the matrix core for 32 clocks, so a read placed
// behind a product issues in its shadow; reads grouped ahead of the products hold the first product up.
template <int CQ>
__device__ __forceinline__ void wide_interleave_reads()
{
#pragma unroll
    for (int c4 = 0; c4 < CQ; ++c4) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // one matrix instruction
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);      // one LDS read
    }
}

// PRE: the folded weights come from `gw`, where a set-up launch of the same call has put them in the order the lanes
// hold them (float index ((tp OB + ob) CQ + VW q) 64 + lane VW + e for the A operand c4 = VW q + e of tap tp): the
// workgroup skips the weight preparation - half the time of a call on 100 images of 48 x 8 x 8 - and needs LDS for
// its rings only.
template <int CQ, int DIR, int MAXW, bool PAD, bool PRE>
__global__ __launch_bounds__(64 * MAXW) void k_solve_wide_reg(const float *__restrict__ in,
                                                              const float *__restrict__ w,
                                                              const float *__restrict__ gw, float *__restrict__ out,
                                                              int H, int W, int NB, float *logdet, int Cr_arg)
{
    static_assert(!(PRE && PAD), "prefolded weights are laid out for whole groups of four channels");
    constexpr int C = 4 * CQ, K = kWideK, NT = K * K, R = kWideRing;
    const int Cr = PAD ? Cr_arg : C;
    constexpr int OB = wide_out_blocks(C), OR = 16 * OB, CPAD = C + 1;
    constexpr int CP = C + wide_vec<CQ>();      // row of the rings: a multiple of the vector width, odd in vectors
    extern __shared__ float smem[];
    const int HP = 16 * NB + K - 1, YR = 16 * NB;
    float *sWt = smem;                          // set-up: [NT][OR][CPAD], then the scratch of the weight preparation
    float *ring = smem;                         // run: [R][HP][CP], permuted channels
    float *ybuf = ring + R * HP * CP;           // run: [2][YR][CP], the input of this and of the next step
    int *sflag = reinterpret_cast<int *>(ybuf + 2 * YR * CP);      // run: [waves] steps finished
    const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int band = wave / OB, ob = wave % OB;
    const int n = lane & 15, g = lane >> 4;

    // this lane's A operands: row m = n -> output channel 16 ob + n, K slot g -> input channel 4 c4 + g
    float wAr[NT][CQ];
    if constexpr (PRE) {
        constexpr int VW = wide_vec<CQ>();
        typedef float wvec_t __attribute__((ext_vector_type(VW)));
        const float *wl = gw + (ob * CQ * 64 + lane * VW);
#pragma unroll
        for (int tp = 0; tp < NT; ++tp)
#pragma unroll
            for (int q = 0; q < CQ / VW; ++q) {
                const wvec_t v = *reinterpret_cast<const wvec_t *>(wl + (tp * OB * CQ + VW * q) * 64);
#pragma unroll
                for (int e = 0; e < VW; ++e)
                    wAr[tp][VW * q + e] = v[e];
            }
    } else {
        wide_fold_weights<CQ, DIR, PAD>(w, sWt, sWt + NT * OR * CPAD, Cr);
        const int a_base = (16 * ob + n) * CPAD + g;
#pragma unroll
        for (int tp = 0; tp < NT; ++tp)
#pragma unroll
            for (int c4 = 0; c4 < CQ; ++c4)
                wAr[tp][c4] = sWt[tp * OR * CPAD + a_base + 4 * c4];
        __syncthreads();
    }
    for (int idx = tid; idx < (R * HP + 2 * YR) * CP + 16; idx += nt)
        ring[idx] = 0.0f;       // (the flags too: zero bits)
    __syncthreads();

    const int r = 16 * band + n;
    const bool row_ok = r < H;
    const size_t img = (size_t)blockIdx.x * Cr * H * W;
    const int b_row = (r + K - 1) * CP + g * CQ;                 // + slot * HP * CP - da * CP
    const int y_row = r * CP + g * CQ;                           // + slot * YR * CP
    const int o_first = 16 * ob + 4 * g;                         // first of this lane's four output channels
    auto gaddr = [&](int ch, int rr, int cc) -> size_t {     // ch < Cr
        return img + ((size_t)(DIR ? Cr - 1 - ch : ch) * H + (DIR ? H - 1 - rr : rr)) * W + (DIR ? W - 1 - cc : cc);
    };
    // the wave's share of the input of step t: channels 16 ob + 4 q + g, q = 0..3, of pixel (r, t - r)
    auto load_y = [&](int t, float (&yv)[4]) {
        const int c = t - r;
        const bool ok = row_ok && (unsigned)c < (unsigned)W;
        const int rr = row_ok ? r : 0, cc = ok ? c : 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int ch = 16 * ob + 4 * q + g;
            const float v = in[gaddr(ch < Cr ? ch : Cr - 1, rr, cc)];
            yv[q] = (ok && ch < Cr) ? v : 0.0f;
        }
    };
    auto store_y = [&](int slot, const float (&yv)[4]) {
        float *dst = ybuf + slot * YR * CP + y_row + 4 * ob;    // channel 16 ob + 4 q + g sits at g CQ + 4 ob + q
        if constexpr (CQ % 4 == 0) {
            *reinterpret_cast<f32x4 *>(dst) = f32x4{yv[0], yv[1], yv[2], yv[3]};
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (4 * ob + q < CQ)
                    dst[q] = yv[q];
        }
    };
    // Small images need few waves for the solve (bands x blocks of output channels) but the set-up above is
    // work for many threads (C^3 multiply-adds per tap), so the launch may bring more waves than the solve
    // uses: they have helped up to here and leave after this barrier, the last one of the kernel.
    const int nw = NB * OB;
    float ynext[4];
    if (wave < nw) {
        load_y(0, ynext);
        store_y(0, ynext);
    }
    __syncthreads();
    if (wave >= nw)
        return;

    // Of the nine taps only three need the step just finished: Linv y (tap 0), (0,1) and (1,0).  The other six
    // read results at least two steps old, so their 6 C/4 products for step t + 1 are issued during step t,
    // AFTER this wave has published its result of step t and BEFORE it needs anybody else's: the waves do not
    // meet at a barrier but raise a flag (step count, one per wave, in LDS) when their result is in the ring
    // and poll the others' flags only when they come back for the three dependent taps - by then the others
    // have long arrived.  No wave is ever more than one step ahead of another (it needs every flag of step
    // t before it starts step t + 1), which is what the five ring slots and the two input slots allow.
    // The polls are bounded (all waves of a workgroup are resident, so the bound is never reached; a wave
    // that reached it would write NaN).
    constexpr int kCrit[3] = {0, 1, 3};
    constexpr int kPre[6] = {2, 4, 5, 6, 7, 8};
    bool lost = false;
    const int nsteps = H + W - 1;
    int tm = 0;                                                 // t mod R
    f32x4 acc0 = f32x4{0.f, 0.f, 0.f, 0.f}, acc1 = f32x4{0.f, 0.f, 0.f, 0.f};    // the six old taps of step 0: zeros
    auto read_tap = [&](int tp, int t, int tmod, float (&ob_)[CQ]) {
        const int da = tp / K, db = tp % K, lag = da + db;
        int slot = tmod - lag;
        slot += slot < 0 ? R : 0;
        const float *bp = tp == 0 ? ybuf + (t & 1) * YR * CP + y_row : ring + slot * HP * CP + b_row - da * CP;
        wide_read_operands<CQ>(bp, ob_);
    };
    for (int t = 0; t < nsteps; ++t) {
        load_y(t + 1, ynext);                                   // one step ahead (past the last step: zeros)
        // ---- everybody's result of step t - 1 (and input of step t) is in LDS
        if (t > 0 && !lost) {
            int spins = 0;
            for (;;) {
                const int v = lane < nw ? __hip_atomic_load(sflag + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) : t;
                if (__builtin_amdgcn_ballot_w64(v < t) == 0)
                    break;
                if (++spins > (1 << 24)) {
                    lost = true;
                    break;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
        }
        float opb[2][CQ];
        read_tap(kCrit[0], t, tm, opb[0]);
#pragma unroll
        for (int q = 0; q < 3; ++q) {
            if (q + 1 < 3)
                read_tap(kCrit[q + 1], t, tm, opb[(q + 1) & 1]);
#pragma unroll
            for (int c4 = 0; c4 < CQ; ++c4) {
                if (c4 & 1)
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(wAr[kCrit[q]][c4], opb[q & 1][c4], acc1, 0, 0, 0);
                else
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(wAr[kCrit[q]][c4], opb[q & 1][c4], acc0, 0, 0, 0);
            }
            wide_interleave_reads<CQ>();
            __builtin_amdgcn_sched_barrier(0);
        }
        // (the first operands of the old taps of step t + 1 are fetched while the result is being stored)
        const int tn = tm + 1 == R ? 0 : tm + 1;
        read_tap(kPre[0], t + 1, tn, opb[0]);
        __builtin_amdgcn_sched_barrier(0);
        f32x4 acc = acc0 + acc1;
        if (lost)
            acc = f32x4{__builtin_nanf(""), __builtin_nanf(""), __builtin_nanf(""), __builtin_nanf("")};
        // The next step's input goes to LDS BEFORE this step's global stores are issued: vector memory operations
        // complete in order, so waiting for the loads behind the stores would wait for the stores' round trip
        // in every step; this way the stores have a whole step to complete.
        store_y((t + 1) & 1, ynext);
        __builtin_amdgcn_sched_barrier(0);
        const int c = t - r;
        const bool ok = row_ok && (unsigned)c < (unsigned)W;
        float *rp = ring + tm * HP * CP + (r + K - 1) * CP;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int ch = o_first + j;
            if (ch < C) {
                rp[(ch & 3) * CQ + (ch >> 2)] = ok ? acc[j] : 0.0f;     // pixels outside the image count as zeros
                if (ok && ch < Cr)
                    out[gaddr(ch, r, c)] = acc[j];
            }
        }
        // ---- published: the LDS writes above are complete before the flag moves
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        if (lane == 0)
            __hip_atomic_store(sflag + wave, t + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        // ---- the six old taps of step t + 1
        acc0 = f32x4{0.f, 0.f, 0.f, 0.f};
        acc1 = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int q = 0; q < 6; ++q) {
            if (q + 1 < 6)
                read_tap(kPre[q + 1], t + 1, tn, opb[(q + 1) & 1]);
#pragma unroll
            for (int c4 = 0; c4 < CQ; ++c4) {
                if (c4 & 1)
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(wAr[kPre[q]][c4], opb[q & 1][c4], acc1, 0, 0, 0);
                else
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(wAr[kPre[q]][c4], opb[q & 1][c4], acc0, 0, 0, 0);
            }
            wide_interleave_reads<CQ>();
            __builtin_amdgcn_sched_barrier(0);
        }
        tm = tn;
    }
    if (logdet && blockIdx.x == 0 && wave == 0)
        wave_logdet_any(w, Cr, K, H, W, logdet);
}

// the rings, the two input slots and the step flags
static size_t wide_reg_run_lds_bytes(int C, int H)
{
    const size_t NB = (H + 15) / 16, CQ = C / 4, CP = C + (CQ % 4 == 0 ? 4 : (CQ % 2 == 0 ? 2 : 1));
    return sizeof(float) * (((size_t)kWideRing * (16 * NB + kWideK - 1) + 2 * 16 * NB) * CP + 16);
}

static size_t wide_reg_lds_bytes(int C, int H)
{
    const size_t NB = (H + 15) / 16, OR = 16 * (size_t)wide_out_blocks(C), CPAD = C + 1;
    const size_t CQ = C / 4, CP = C + (CQ % 4 == 0 ? 4 : (CQ % 2 == 0 ? 2 : 1));
    const size_t setup = (size_t)kWideK * kWideK * OR * CPAD + wide_fold_scratch_floats(C);
    const size_t run = ((size_t)kWideRing * (16 * NB + kWideK - 1) + 2 * 16 * NB) * CP + 16;
    return sizeof(float) * (setup > run ? setup : run);
}

// at most eight waves: each may use 256 registers; at most twelve: 168, which the weights of up to 48 channels
// still fit (48 channels leave three values of the set-up in scratch memory)
static bool wide_reg_supported(int C, int H)
{
    return ((H + 15) / 16) * wide_out_blocks(C) <= 12 && wide_reg_lds_bytes(C, H) <= kMaxLdsBytes;
}

template <int CQ, int MAXW, bool PAD>
static int launch_wide_reg(int dir, const float *in, const float *w, float *out, int B, int Cr, int H, int W,
                           hipStream_t stream, float *logdet, float *gw)
{
    constexpr int C = 4 * CQ;
    const int NB = (H + 15) / 16;
    if constexpr (!PAD) {
        if (gw) {
            // the weights folded once for the call by a launch of their own, the solve with the waves it needs
            if (int s = launch_wide_fold(dir, w, gw, C, kWideK, stream))
                return s;
            const size_t lds = wide_reg_run_lds_bytes(C, H);
            const void *fn = dir ? reinterpret_cast<const void *>(&k_solve_wide_reg<CQ, 1, MAXW, false, true>)
                                 : reinterpret_cast<const void *>(&k_solve_wide_reg<CQ, 0, MAXW, false, true>);
            if (!ensure_dynamic_lds(fn, lds))
                return INVCONV_ERR_UNSUPPORTED;
            const dim3 block((unsigned)(64 * NB * wide_out_blocks(C)));
            if (dir)
                hipLaunchKernelGGL((k_solve_wide_reg<CQ, 1, MAXW, false, true>), dim3(B), block, lds, stream, in, w, gw,
                                   out, H, W, NB, logdet, Cr);
            else
                hipLaunchKernelGGL((k_solve_wide_reg<CQ, 0, MAXW, false, true>), dim3(B), block, lds, stream, in, w, gw,
                                   out, H, W, NB, logdet, Cr);
            return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
        }
    }
    const size_t lds = wide_reg_lds_bytes(C, H);
    const void *fn = dir ? reinterpret_cast<const void *>(&k_solve_wide_reg<CQ, 1, MAXW, PAD, false>)
                         : reinterpret_cast<const void *>(&k_solve_wide_reg<CQ, 0, MAXW, PAD, false>);
    if (!ensure_dynamic_lds(fn, lds))
        return INVCONV_ERR_UNSUPPORTED;
    // up to one workgroup per compute unit: eight waves at least, the ones the solve does not use help with the
    // set-up (48 x 8 x 8, B = 100: 70 -> 50 us); more workgroups than that are better off with more of them resident
    // (48 channels: the set-up's LDS leaves room for one workgroup per compute unit whatever the batch)
    int waves = NB * wide_out_blocks(C);
    if ((B <= 256 || 2 * lds > kMaxLdsBytes) && waves < 8)
        waves = 8 < MAXW ? 8 : MAXW;
    const dim3 block((unsigned)(64 * waves));
    if (dir)
        hipLaunchKernelGGL((k_solve_wide_reg<CQ, 1, MAXW, PAD, false>), dim3(B), block, lds, stream, in, w,
                           (const float *)nullptr, out, H, W, NB, logdet, Cr);
    else
        hipLaunchKernelGGL((k_solve_wide_reg<CQ, 0, MAXW, PAD, false>), dim3(B), block, lds, stream, in, w,
                           (const float *)nullptr, out, H, W, NB, logdet, Cr);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

static size_t wide_lds_bytes(int C, int H)
{
    const size_t NB = (H + 15) / 16, OR = 16 * (size_t)wide_out_blocks(C), CPAD = C + 1;
    const size_t ring = (size_t)kWideRing * (16 * NB + kWideK - 1) * CPAD, scratch = wide_fold_scratch_floats(C);
    return sizeof(float) * ((size_t)kWideK * kWideK * OR * CPAD + (ring > scratch ? ring : scratch));
}

// Channel counts that are no multiple of 4 run the next multiple with the surplus channels switched off.
bool wide_supported(int C, int H, int k)
{
    const int Cp = (C + 3) / 4 * 4;
    return k == kWideK && C >= 17 && C <= 48 && ((H + 15) / 16) * wide_out_blocks(Cp) <= 16 &&
           wide_lds_bytes(Cp, H) <= kMaxLdsBytes;
}

template <int CQ, bool PAD>
static int launch_wide_cq(int dir, const float *in, const float *w, float *out, int B, int Cr, int H, int W,
                          hipStream_t stream, float *logdet, float *gw)
{
    constexpr int C = 4 * CQ;
    const int NB = (H + 15) / 16;
    if (wide_reg_supported(C, H))
        return NB * wide_out_blocks(C) <= 8
                   ? launch_wide_reg<CQ, 8, PAD>(dir, in, w, out, B, Cr, H, W, stream, logdet, gw)
                   : launch_wide_reg<CQ, 12, PAD>(dir, in, w, out, B, Cr, H, W, stream, logdet, gw);
    const size_t lds = wide_lds_bytes(C, H);
    const void *fn = dir ? reinterpret_cast<const void *>(&k_solve_wide<CQ, 1, PAD>)
                         : reinterpret_cast<const void *>(&k_solve_wide<CQ, 0, PAD>);
    if (!ensure_dynamic_lds(fn, lds))
        return INVCONV_ERR_UNSUPPORTED;
    const dim3 block((unsigned)(64 * NB * wide_out_blocks(C)));
    if (dir)
        hipLaunchKernelGGL((k_solve_wide<CQ, 1, PAD>), dim3(B), block, lds, stream, in, w, out, H, W, NB, logdet, Cr);
    else
        hipLaunchKernelGGL((k_solve_wide<CQ, 0, PAD>), dim3(B), block, lds, stream, in, w, out, H, W, NB, logdet, Cr);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

// bytes of scratch with which the weights are folded once per call instead of once per workgroup (0: not for this shape)
size_t wide_prefold_ws_bytes(int C, int H, int k)
{
    return wide_supported(C, H, k) && C % 4 == 0 && C >= 20 && wide_reg_supported(C, H) ? wide_stream_ws_bytes(C, k) : 0;
}

// gw: null, or wide_prefold_ws_bytes(C, H, k) > 0 bytes of device scratch, 256-byte aligned
int launch_solve_wide(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W, int k,
                      hipStream_t stream, float *logdet, float *gw)
{
    if (gw && !wide_prefold_ws_bytes(C, H, k))
        gw = nullptr;
    if (!wide_supported(C, H, k))
        return INVCONV_ERR_VARIANT;
    auto by_cq = [&](auto pad_tag) -> int {
        constexpr bool PAD = decltype(pad_tag)::value;
        switch ((C + 3) / 4) {
        case 5: return launch_wide_cq<5, PAD>(dir, in, w, out, B, C, H, W, stream, logdet, gw);
        case 6: return launch_wide_cq<6, PAD>(dir, in, w, out, B, C, H, W, stream, logdet, gw);
        case 7: return launch_wide_cq<7, PAD>(dir, in, w, out, B, C, H, W, stream, logdet, gw);
        case 8: return launch_wide_cq<8, PAD>(dir, in, w, out, B, C, H, W, stream, logdet, gw);
        case 9: return launch_wide_cq<9, PAD>(dir, in, w, out, B, C, H, W, stream, logdet, gw);
        case 10: return launch_wide_cq<10, PAD>(dir, in, w, out, B, C, H, W, stream, logdet, gw);
        case 11: return launch_wide_cq<11, PAD>(dir, in, w, out, B, C, H, W, stream, logdet, gw);
        case 12: return launch_wide_cq<12, PAD>(dir, in, w, out, B, C, H, W, stream, logdet, gw);
        default: return INVCONV_ERR_VARIANT;
        }
    };
    return C % 4 ? by_cq(std::true_type()) : by_cq(std::false_type());
}

}  // namespace invconv
