// Wavefront solve for many channels (C = 20 .. 48, a multiple of 4) with the OTHER kernel sizes of the paper's
// kernel-size ablation (k = 2, 5, 7, 9, 11): the shapes its model reaches after two squeezes (Section 4.1) when
// the kernel is not 3 x 3.  gfx950 only.
//
// Same scheme as the 3 x 3 many-channel kernel: folded weights (Linv = inverse of the current-pixel block,
// Cf_tap = Linv W_tap, so x_p = Linv y_p - sum_tap Cf_tap x_{p - tap}: Eq. 1 rearranged), one workgroup per image,
// wave (band, ob) owns rows 16 band .. and output channels 16 ob .., all rows in lock step, the results of the
// last 2k - 1 steps in an LDS ring, one tap = C/4 v_mfma_f32_16x16x4_f32 with a weight tile as A operand and the
// ring as B operand, one LDS-only barrier per step.
// What differs: k^2 C^2 folded weights (230 KB at 48 channels and k = 5, 1.1 MB at k = 11) fit neither LDS nor
// a workgroup's registers, so a set-up launch folds them ONCE per call into the caller's workspace, laid out as the
// waves read them - 64 consecutive floats per (tap, block of output channels, group of four input channels) - and
// every wave streams its A operands from there (L2 hits after the first workgroup), one row of taps ahead of the
// matrix instructions that use them.  Without a workspace these shapes keep the per-diagonal fallback.
#include "invconv_common.h"
#include "invconv_launch.h"
#include "invconv_tri_inverse.h"

namespace invconv {

typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

__host__ __device__ constexpr int ws_out_blocks(int C) { return (C + 15) / 16; }

// A lane fetches VW = 4, 2 or 1 consecutive A operands (input-channel groups c4 = VW q .. VW q + VW - 1) with one
// load: few, wide loads keep the number of fetches in flight below what a wave may have outstanding.
__host__ __device__ constexpr int ws_vec(int CQ) { return CQ % 4 == 0 ? 4 : (CQ % 2 == 0 ? 2 : 1); }

// gw[(((tp OB + ob) CQ/VW + q) 64 + lane) VW + e] = A operand of lane (n, g) = (lane % 16, lane / 16) for c4 = VW q + e:
// entry [16 ob + n][4 c4 + g] of Linv (tp = 0) or of -Linv W_tp; rows past C are zeros.  One workgroup per tap.
template <int CQ, int DIR>
__global__ __launch_bounds__(1024) void k_wide_fold_stream(const float *__restrict__ w, float *__restrict__ gw, int K)
{
    constexpr int C = 4 * CQ;
    extern __shared__ __attribute__((aligned(16))) float fs[];
    float *sL = fs, *sLinv = sL + C * C, *sT = sLinv + C * C;
    const int tid = threadIdx.x, tp = blockIdx.x;
    auto entry = [&](int t, int o, int i) -> float {       // oriented, masked entry (t, o, i)
        const int a = K - 1 - t / K, b = K - 1 - t % K;
        const int oo = DIR ? C - 1 - i : o, ii = DIR ? C - 1 - o : i;
        const float v = w[((oo * C + ii) * K + a) * K + b];
        return (t == 0 && ii > oo) ? 0.0f : v;
    };
    {
        // all of a thread's entries in flight before the first goes to LDS
        constexpr int NL = (C * C + 1023) / 1024;
        float a[NL], t[NL];
#pragma unroll
        for (int u = 0; u < NL; ++u) {
            const int idx = tid + 1024 * u;
            const bool ok = idx < C * C;
            const int o = ok ? idx / C : 0, i = ok ? idx % C : 0;
            a[u] = entry(0, o, i);
            t[u] = tp ? entry(tp, o, i) : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < NL; ++u) {
            const int idx = tid + 1024 * u;
            if (idx < C * C) {
                sL[idx] = a[u];
                sT[idx] = t[u];
            }
        }
    }
    __syncthreads();
    // Linv in 16 x 16 blocks by the whole workgroup
    tri_inverse_blocks<C>(sL, sLinv, C, sT + C * C);
    constexpr int OB = ws_out_blocks(C);
    float *dst = gw + (size_t)tp * OB * CQ * 64;
    constexpr int VW = ws_vec(CQ);
    if (tp == 0) {
        for (int idx = tid; idx < OB * CQ * 64; idx += 1024) {
            const int e = idx % VW, lane = (idx / VW) & 63, q = (idx / (VW * 64)) % (CQ / VW), ob = idx / (CQ * 64);
            const int o = 16 * ob + (lane & 15), i = 4 * (VW * q + e) + (lane >> 4);
            dst[idx] = o < C ? sLinv[o * C + i] : 0.0f;
        }
        return;
    }
    // -Linv W_tp on the matrix cores: a task is one 16 x 16 block of the product, a wave per task; Linv is lower
    // triangular, so a block of rows 16 ob .. needs only the first 4 (ob + 1) of the C/4 instructions.  Rows past C
    // are written as zeros.
    const int wave = tid >> 6, lane = tid & 63, n = lane & 15, g = lane >> 4;
    for (int task = wave; task < OB * OB; task += 16) {
        const int ob = task / OB, ib = task % OB;
        const int o_a = 16 * ob + n, i_b = 16 * ib + n;
        const int nc = 4 * (ob + 1) < CQ ? 4 * (ob + 1) : CQ;
        f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int c = 0; c < nc; ++c) {
            const float av = sLinv[(o_a < C ? o_a : 0) * C + 4 * c + g];
            const float bv = sT[(4 * c + g) * C + (i_b < C ? i_b : 0)];
            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(o_a < C ? av : 0.0f, i_b < C ? bv : 0.0f, acc, 0, 0, 0);
        }
        if (i_b < C) {
            const int c4 = i_b >> 2, gi = i_b & 3;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int m = 4 * g + j;        // row 16 ob + m of the product, held by lane (m, gi) of wave ob
                dst[ob * CQ * 64 + ((c4 / VW) * 64 + m + 16 * gi) * VW + c4 % VW] = -acc[j];
            }
        }
    }
}

// Taps are taken in groups of D whose A operands sit in registers one group ahead: a row of taps (D = K, group =
// da, member = db) for k >= 5, all four taps for k = 2.
template <int K>
__host__ __device__ constexpr int ws_group() { return K == 2 ? 4 : K; }

template <int CQ, int K, int DIR>
__global__ __launch_bounds__(256) void k_solve_wide_stream(const float *__restrict__ in, const float *__restrict__ gw,
                                                          float *__restrict__ out, int B, int H, int W, int NB,
                                                          int pack)
{
    constexpr int C = 4 * CQ, NT = K * K, R = 2 * K - 1, D = ws_group<K>(), G = NT / D;
    constexpr int OB = ws_out_blocks(C), CPAD = C + 1;
    static_assert(NT % D == 0, "whole groups of taps");
    extern __shared__ float smem[];
    // pack (images of at most 8 rows): a workgroup takes TWO images, rows n = 0 .. 7 of the 16 pixel columns of an
    // instruction are the first image's rows and n = 8 .. 15 the second's (half of every product was padding
    // otherwise); in the ring each image has its own K - 1 rows of zeros on top.
    const int HP = 16 * NB + (pack ? 2 : 1) * (K - 1);
    float *ring = smem;                         // [R][HP][CPAD]: x of the last R steps, K - 1 rows of zeros on top
    const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int band = wave / OB, ob = wave % OB;
    const int n = lane & 15, g = lane >> 4;
    for (int idx = tid; idx < R * HP * CPAD; idx += nt)
        ring[idx] = 0.0f;

    const int second = pack ? n >> 3 : 0;                        // which of the workgroup's images
    const int r = pack ? (n & 7) : 16 * band + n;                // row in the image
    const int image = pack ? 2 * (int)blockIdx.x + second : (int)blockIdx.x;
    const bool row_ok = r < H && image < B;
    const size_t img = (size_t)(image < B ? image : B - 1) * C * H * W;
    const int ring_row = (pack ? 8 * second + r : r) + (K - 1) * (1 + second);
    const int b_row = ring_row * CPAD + g;                       // + slot * HP * CPAD - da * CPAD + 4 c4
    const int o_first = 16 * ob + 4 * g;                         // first of this lane's four output channels
    auto gaddr = [&](int ch, int rr, int cc) -> size_t {
        return img + ((size_t)(DIR ? C - 1 - ch : ch) * H + (DIR ? H - 1 - rr : rr)) * W + (DIR ? W - 1 - cc : cc);
    };
    auto load_y = [&](int t, float (&yv)[CQ]) {
        const int c = t - r;
        const bool ok = row_ok && (unsigned)c < (unsigned)W;
        const int rr = row_ok ? r : 0, cc = ok ? c : 0;
#pragma unroll
        for (int c4 = 0; c4 < CQ; ++c4) {
            const float v = in[gaddr(4 * c4 + g, rr, cc)];
            yv[c4] = ok ? v : 0.0f;
        }
    };
    // this wave's A operands of tap tp: VW consecutive floats per lane and load, at float index
    // tp kTapStride + ob CQ 64 + q 64 VW + lane VW. Buffer loads: the lane's part of the address is one constant
    // 32-bit register and the rest a scalar. (A load with a 64-bit address per lane holds up the wave's next matrix
    // instruction for some 20 clocks whatever its width, a buffer load for about 5: measured with 12 products and
    // 3 loads in turn, 37.9 against 33.6 clocks per product, 32.4 without loads.)
    constexpr int VW = ws_vec(CQ);
    constexpr int kTapStride = OB * CQ * 64;
    const __amdgpu_buffer_rsrc_t wrsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(gw), 0, K * K * kTapStride * (int)sizeof(float), 0x00020000);
    const int wlane = lane * VW * (int)sizeof(float);
    const int wblock = ob * CQ * 64 * (int)sizeof(float);
    float aw[D][CQ];
    auto fetch_tap = [&](int tp, float (&dst)[CQ]) {
#pragma unroll
        for (int q = 0; q < CQ / VW; ++q) {
            const int soff = (tp * kTapStride + q * 64 * VW) * (int)sizeof(float) + wblock;
            if constexpr (VW == 4) {
                const f32x4 v = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, wlane, soff, 0));
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    dst[4 * q + e] = v[e];
            } else if constexpr (VW == 2) {
                typedef float f32x2 __attribute__((ext_vector_type(2)));
                const f32x2 v = __builtin_bit_cast(f32x2, __builtin_amdgcn_raw_buffer_load_b64(wrsrc, wlane, soff, 0));
                dst[2 * q] = v[0];
                dst[2 * q + 1] = v[1];
            } else {
                dst[q] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(wrsrc, wlane, soff, 0));
            }
        }
    };
#pragma unroll
    for (int u = 0; u < D; ++u)
        fetch_tap(u, aw[u]);
    float ycur[CQ], ynext[CQ];
    load_y(0, ycur);
    __syncthreads();        // ring zeroed

    const int nsteps = H + W - 1;
    int tm = 0;                                                 // t mod R
    for (int t = 0; t < nsteps; ++t) {
        load_y(t + 1, ynext);                                   // one step ahead (past the last step: zeros)
        // four accumulators in turn, summed at the end of the step
        f32x4 accs[4];
#pragma unroll
        for (int q = 0; q < 4; ++q)
            accs[q] = f32x4{0.f, 0.f, 0.f, 0.f};
        // B operands of tap (grp, u): the ring slot of lag da + db, da rows up (tap (0, 0) takes the input y of the
        // step instead: the term Linv y)
        auto read_b = [&](int grp, int u, float (&o)[CQ]) {
            const int da = D == K ? grp : u / K, db = D == K ? u : u % K, lag = da + db;
            int slot = tm - lag;
            slot += slot < 0 ? R : 0;
            const float *bp = ring + slot * HP * CPAD + b_row - da * CPAD;
#pragma unroll
            for (int c4 = 0; c4 < CQ; ++c4)
                o[c4] = bp[4 * c4];
        };
        // The operands of the NEXT tap are read from LDS while the matrix cores work on the current one: two
        // buffers taken in turn; a group of an odd number of taps ends on the buffer the next group starts with,
        // so its last tap reads ahead into the other one and hands over with one copy per group. A wave issues in
        // order and a product occupies the matrix core for 32 clocks: every other instruction of a tap (LDS reads,
        // weight fetches) is placed BETWEEN two products, where it issues in the shadow of the one before it -
        // grouped ahead of the products they cost 150 clocks per tap on top of the products' 384.
        float opb[2][CQ];
#pragma unroll
        for (int c4 = 0; c4 < CQ; ++c4)
            opb[0][c4] = ycur[c4];
#pragma unroll 1
        for (int grp = 0; grp < G; ++grp) {
            const int gnext = grp + 1 == G ? 0 : grp + 1;       // (the last group fetches the first one of the next step)
#pragma unroll
            for (int u = 0; u < D; ++u) {
                constexpr int kLast = D - 1;
                if (u < kLast)
                    read_b(grp, u + 1, opb[(u + 1) & 1]);
                else
                    read_b(gnext, 0, opb[(kLast & 1) ^ 1]);     // (after the last tap of the step: read and dropped)
#pragma unroll
                for (int c4 = 0; c4 < CQ; ++c4)
                    accs[c4 & 3] = __builtin_amdgcn_mfma_f32_16x16x4f32(aw[u][c4], opb[u & 1][c4], accs[c4 & 3], 0, 0, 0);
                // the same member of the next group takes the registers just used (a single group, k = 2, stays)
                if constexpr (G > 1)
                    fetch_tap(gnext * D + u, aw[u]);
                // issue order of the tap: product, LDS read, product, LDS read, ...; each weight fetch after the
                // last product that reads the registers it overwrites
#pragma unroll
                for (int c4 = 0; c4 < CQ; ++c4) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // one matrix instruction
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);      // one LDS read
                    if (G > 1 && (c4 + 1) % VW == 0)
                        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // one vector memory read
                }
                __builtin_amdgcn_sched_barrier(0);
                if (u == kLast && ((kLast & 1) ^ 1) != 0) {
#pragma unroll
                    for (int c4 = 0; c4 < CQ; ++c4)
                        opb[0][c4] = opb[1][c4];
                }
            }
        }
        const f32x4 acc = (accs[0] + accs[1]) + (accs[2] + accs[3]);
#pragma unroll
        for (int c4 = 0; c4 < CQ; ++c4)
            ycur[c4] = ynext[c4];
        const int c = t - r;
        const bool ok = row_ok && (unsigned)c < (unsigned)W;
        float *rp = ring + tm * HP * CPAD + ring_row * CPAD + o_first;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (o_first + j < C) {
                rp[j] = ok ? acc[j] : 0.0f;                     // pixels outside the image count as zeros
                if (ok)
                    out[gaddr(o_first + j, r, c)] = acc[j];
            }
        }
        tm = tm + 1 == R ? 0 : tm + 1;
        // workgroup barrier that orders LDS only: the global stores and the weight fetches stay in flight across it
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    }
}

size_t ws_ring_bytes(int C, int H, int k)
{
    const size_t NB = (H + 15) / 16;
    return sizeof(float) * (size_t)(2 * k - 1) * (16 * NB + (H <= 8 ? 2 : 1) * (k - 1)) * (C + 1);
}

template <int CQ, int K>
int launch_stream_ck(int dir, const float *in, const float *gw, float *out, int B, int H, int W, hipStream_t stream)
{
    const int NB = (H + 15) / 16;
    const size_t lds = ws_ring_bytes(4 * CQ, H, K);
    const void *fn = dir ? reinterpret_cast<const void *>(&k_solve_wide_stream<CQ, K, 1>)
                         : reinterpret_cast<const void *>(&k_solve_wide_stream<CQ, K, 0>);
    if (!ensure_dynamic_lds(fn, lds))
        return INVCONV_ERR_UNSUPPORTED;
    const dim3 block((unsigned)(64 * NB * ws_out_blocks(4 * CQ)));
    const int pack = H <= 8 ? 1 : 0;
    const dim3 grid((unsigned)(pack ? (B + 1) / 2 : B));
    if (dir)
        hipLaunchKernelGGL((k_solve_wide_stream<CQ, K, 1>), grid, block, lds, stream, in, gw, out, B, H, W, NB, pack);
    else
        hipLaunchKernelGGL((k_solve_wide_stream<CQ, K, 0>), grid, block, lds, stream, in, gw, out, B, H, W, NB, pack);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

template <int CQ>
int launch_fold_cq(int dir, const float *w, float *gw, int k, hipStream_t stream)
{
    const size_t flds = sizeof(float) * (3 * (size_t)(4 * CQ) * (4 * CQ) + tri_inverse_tmp_floats());
    if (dir)
        hipLaunchKernelGGL((k_wide_fold_stream<CQ, 1>), dim3(k * k), dim3(1024), flds, stream, w, gw, k);
    else
        hipLaunchKernelGGL((k_wide_fold_stream<CQ, 0>), dim3(k * k), dim3(1024), flds, stream, w, gw, k);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

template <int CQ>
int launch_stream_cq(int dir, const float *in, const float *w, float *gw, float *out, int B, int H, int W, int k,
                     hipStream_t stream)
{
    if (int s = launch_fold_cq<CQ>(dir, w, gw, k, stream))
        return s;
    switch (k) {
    case 2: return launch_stream_ck<CQ, 2>(dir, in, gw, out, B, H, W, stream);
    case 5: return launch_stream_ck<CQ, 5>(dir, in, gw, out, B, H, W, stream);
    case 7: return launch_stream_ck<CQ, 7>(dir, in, gw, out, B, H, W, stream);
    case 9: return launch_stream_ck<CQ, 9>(dir, in, gw, out, B, H, W, stream);
    case 11: return launch_stream_ck<CQ, 11>(dir, in, gw, out, B, H, W, stream);
    default: return INVCONV_ERR_VARIANT;
    }
}

}  // namespace

// at most four waves (bands x blocks of 16 output channels), the ring in LDS
bool wide_stream_supported(int C, int H, int k)
{
    const bool kk = k == 2 || k == 5 || k == 7 || k == 9 || k == 11;
    return kk && C % 4 == 0 && C >= 20 && C <= 48 && ((H + 15) / 16) * ws_out_blocks(C) <= 4 &&
           ws_ring_bytes(C, H, k) <= kMaxLdsBytes;
}

// bytes of workspace the folded weights take
size_t wide_stream_ws_bytes(int C, int k)
{
    return sizeof(float) * (size_t)k * k * ws_out_blocks(C) * (C / 4) * 64;
}

// The set-up launch alone: C = 20 .. 48 in multiples of 4, any k; fills wide_stream_ws_bytes(C, k) bytes at `gw`.
int launch_wide_fold(int dir, const float *w, float *gw, int C, int k, hipStream_t stream)
{
    if (C % 4 || C < 20 || C > 48 || !gw)
        return INVCONV_ERR_VARIANT;
    switch (C / 4) {
    case 5: return launch_fold_cq<5>(dir, w, gw, k, stream);
    case 6: return launch_fold_cq<6>(dir, w, gw, k, stream);
    case 7: return launch_fold_cq<7>(dir, w, gw, k, stream);
    case 8: return launch_fold_cq<8>(dir, w, gw, k, stream);
    case 9: return launch_fold_cq<9>(dir, w, gw, k, stream);
    case 10: return launch_fold_cq<10>(dir, w, gw, k, stream);
    case 11: return launch_fold_cq<11>(dir, w, gw, k, stream);
    case 12: return launch_fold_cq<12>(dir, w, gw, k, stream);
    default: return INVCONV_ERR_VARIANT;
    }
}

// `gw`: wide_stream_ws_bytes(C, k) bytes of device scratch, 256-byte aligned
int launch_solve_wide_stream(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W, int k,
                             hipStream_t stream, float *gw)
{
    if (!wide_stream_supported(C, H, k) || !gw)
        return INVCONV_ERR_VARIANT;
    switch (C / 4) {
    case 5: return launch_stream_cq<5>(dir, in, w, gw, out, B, H, W, k, stream);
    case 6: return launch_stream_cq<6>(dir, in, w, gw, out, B, H, W, k, stream);
    case 7: return launch_stream_cq<7>(dir, in, w, gw, out, B, H, W, k, stream);
    case 8: return launch_stream_cq<8>(dir, in, w, gw, out, B, H, W, k, stream);
    case 9: return launch_stream_cq<9>(dir, in, w, gw, out, B, H, W, k, stream);
    case 10: return launch_stream_cq<10>(dir, in, w, gw, out, B, H, W, k, stream);
    case 11: return launch_stream_cq<11>(dir, in, w, gw, out, B, H, W, k, stream);
    case 12: return launch_stream_cq<12>(dir, in, w, gw, out, B, H, W, k, stream);
    default: return INVCONV_ERR_VARIANT;
    }
}

}  // namespace invconv
