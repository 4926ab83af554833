// Wavefront solve for many channels (C = 20 .. 48, a multiple of 4; k = 3): the shapes a flow reaches after
// two squeezes (Section 4.1).  gfx950 only.
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

namespace invconv {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWideK = 3;
constexpr int kWideRing = 2 * kWideK - 1;

__host__ __device__ constexpr int wide_out_blocks(int C) { return (C + 15) / 16; }

template <int CQ, int DIR>
__global__ __launch_bounds__(1024) void k_solve_wide(const float *__restrict__ in, const float *__restrict__ w,
                                                    float *__restrict__ out, int H, int W, int NB)
{
    constexpr int C = 4 * CQ, K = kWideK, NT = K * K, R = kWideRing;
    constexpr int OB = wide_out_blocks(C), OR = 16 * OB, CPAD = C + 1;
    extern __shared__ float smem[];
    const int HP = 16 * NB + K - 1;
    float *sWt = smem;                          // [NT][OR][CPAD]: tap 0 = Linv, the others = -Linv W_tap
    float *ring = sWt + NT * OR * CPAD;         // [R][HP][CPAD]
    float *sL = ring, *sLinv = ring + C * C;    // folding scratch, dead before the ring is used
    float *sTap = ring + 2 * C * C;             // one oriented tap block at a time
    const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int band = wave / OB, ob = wave % OB;
    const int n = lane & 15, g = lane >> 4;

    // ---- weight preparation (oriented, masked kernel entries straight from global memory)
    auto entry = [&](int tp, int o, int i) -> float {
        const int a = K - 1 - tp / K, b = K - 1 - tp % K;
        const int oo = DIR ? C - 1 - i : o, ii = DIR ? C - 1 - o : i;
        const float v = w[((oo * C + ii) * K + a) * K + b];
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
    for (int tp = 0; tp < NT; ++tp) {
        if (tp > 0) {
            for (int idx = tid; idx < C * C; idx += nt)
                sTap[idx] = entry(tp, idx / C, idx % C);
            __syncthreads();
        }
        for (int idx = tid; idx < OR * CPAD; idx += nt) {
            const int i = idx % CPAD, o = idx / CPAD;
            float v = 0.0f;
            if (o < C && i < C) {
                if (tp == 0) {
                    v = sLinv[o * C + i];
                } else {
                    float s = 0.0f;
                    for (int j = 0; j <= o; ++j)
                        s += sLinv[o * C + j] * sTap[j * C + i];
                    v = -s;
                }
            }
            sWt[tp * OR * CPAD + idx] = v;
        }
        __syncthreads();
    }
    for (int idx = tid; idx < R * HP * CPAD; idx += nt)
        ring[idx] = 0.0f;
    __syncthreads();

    // ---- this lane: pixel row r (B operand column n), input channels 4 c4 + g (K slot g),
    //      A operand row m = n -> output channel 16 ob + n; results: output channels 16 ob + 4 g + j
    const int r = 16 * band + n;
    const bool row_ok = r < H;
    const size_t img = (size_t)blockIdx.x * C * H * W;
    const int a_base = (16 * ob + n) * CPAD + g;                 // + tp * OR * CPAD + 4 c4
    const int b_row = (r + K - 1) * CPAD + g;                    // + slot * HP * CPAD - da * CPAD + 4 c4
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
        const int c = t - r;
        const bool ok = row_ok && (unsigned)c < (unsigned)W;
        float *rp = ring + tm * HP * CPAD + (r + K - 1) * CPAD + o_first;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (o_first + j < C) {
                rp[j] = ok ? acc[j] : 0.0f;                     // pixels outside the image count as zeros
                if (ok)
                    out[gaddr(o_first + j, r, c)] = acc[j];
            }
        }
#pragma unroll
        for (int c4 = 0; c4 < CQ; ++c4)
            ycur[c4] = ynext[c4];
        tm = tm + 1 == R ? 0 : tm + 1;
        // workgroup barrier that orders LDS only: the global loads of the next step's input and this step's
        // global stores stay in flight across it (a full __syncthreads() would wait for them at every step)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    }
}

static size_t wide_lds_bytes(int C, int H)
{
    const size_t NB = (H + 15) / 16, OR = 16 * (size_t)wide_out_blocks(C), CPAD = C + 1;
    const size_t ring = (size_t)kWideRing * (16 * NB + kWideK - 1) * CPAD, scratch = 3 * (size_t)C * C;
    return sizeof(float) * ((size_t)kWideK * kWideK * OR * CPAD + (ring > scratch ? ring : scratch));
}

bool wide_supported(int C, int H, int k)
{
    return k == kWideK && C % 4 == 0 && C >= 20 && C <= 48 && ((H + 15) / 16) * wide_out_blocks(C) <= 16 &&
           wide_lds_bytes(C, H) <= kMaxLdsBytes;
}

template <int CQ>
static int launch_wide_cq(int dir, const float *in, const float *w, float *out, int B, int H, int W, hipStream_t stream)
{
    constexpr int C = 4 * CQ;
    const int NB = (H + 15) / 16;
    const size_t lds = wide_lds_bytes(C, H);
    const void *fn = dir ? reinterpret_cast<const void *>(&k_solve_wide<CQ, 1>)
                         : reinterpret_cast<const void *>(&k_solve_wide<CQ, 0>);
    if (!ensure_dynamic_lds(fn, lds))
        return INVCONV_ERR_UNSUPPORTED;
    const dim3 block((unsigned)(64 * NB * wide_out_blocks(C)));
    if (dir)
        hipLaunchKernelGGL((k_solve_wide<CQ, 1>), dim3(B), block, lds, stream, in, w, out, H, W, NB);
    else
        hipLaunchKernelGGL((k_solve_wide<CQ, 0>), dim3(B), block, lds, stream, in, w, out, H, W, NB);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

int launch_solve_wide(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W, int k,
                      hipStream_t stream)
{
    if (!wide_supported(C, H, k))
        return INVCONV_ERR_VARIANT;
    switch (C / 4) {
    case 5: return launch_wide_cq<5>(dir, in, w, out, B, H, W, stream);
    case 6: return launch_wide_cq<6>(dir, in, w, out, B, H, W, stream);
    case 7: return launch_wide_cq<7>(dir, in, w, out, B, H, W, stream);
    case 8: return launch_wide_cq<8>(dir, in, w, out, B, H, W, stream);
    case 9: return launch_wide_cq<9>(dir, in, w, out, B, H, W, stream);
    case 10: return launch_wide_cq<10>(dir, in, w, out, B, H, W, stream);
    case 11: return launch_wide_cq<11>(dir, in, w, out, B, H, W, stream);
    case 12: return launch_wide_cq<12>(dir, in, w, out, B, H, W, stream);
    default: return INVCONV_ERR_VARIANT;
    }
}

}  // namespace invconv
