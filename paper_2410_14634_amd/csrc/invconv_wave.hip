// Wave-synchronous ("systolic") wavefront solve for few channels (C <= 4),
// images of at most 64 rows.  gfx950 only.
//
// One 64-lane wave solves one image; lane r owns image row r.  At step t lane
// r computes pixel (r, c = t - r), so at every step the wave holds one
// anti-diagonal (Section 3.3: pixels of an anti-diagonal are independent) and
// the whole dependency structure lives in registers:
//   * the pixel's own row, columns c-1 .. c-(k-1), is the lane's history xh;
//   * everything the rows above contribute to pixel (r,c) arrives as one
//     message from lane r-1 (a DPP shift by one lane, no LDS, no barrier).
// Lane r, after computing x(r,c), sends down k-1 partial sums: T[a] is the
// total contribution of rows <= r to pixel (r+a, c).  It is built as
// T[a] = S[a+1] + (row r's own taps), S[.] being what the lane received, so a
// contribution from a rows above travels a hops, one hop per step, and arrives
// exactly when lane r+a reaches column c.
//
// With folded weights (Linv, Cf) the channels of a pixel are independent, so a
// pixel's C outputs are the rows of a 4 x 1 times 1 x 1 outer-product update:
// v_mfma_f32_4x4x1 with lane = pixel (its B operand is the lane's scalar
// history value, its A operand the weight column indexed by lane%4, and its
// four result registers are the pixel's output channels).
#include "invconv_common.h"
#include "invconv_launch.h"

namespace invconv {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// value of the lane above (lane 0 receives 0)
__device__ __forceinline__ float from_lane_above(float v)
{
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x138 /* wave_shr:1 */, 0xf, 0xf, true));
}

constexpr int kWavePF = 16;   // steps of load prefetch

template <int C, int K, int DIR>
__global__ __launch_bounds__(64) void k_solve_wave(const float *__restrict__ in, const float *__restrict__ w,
                                                  float *__restrict__ out, int H, int W)
{
    static_assert(C >= 1 && C <= 4, "one 4-row MFMA block per pixel");
    __shared__ float sL[C * C], sLinv[C * C], sCf[K * K * C * C];
    __shared__ float sA[K * K * C * 4];   // -Cf[tp][o][i] stored as [tp][i][o padded to 4]
    __shared__ float sLi[C * 4];          // Linv[o][j] stored as [j][o padded to 4]

    // All 64 lanes stay active to the end: the matrix instruction reads its weight
    // operand from every lane of a 4-lane block, whatever the execution mask says.
    // Lanes past the last row compute on clamped inputs and never store.
    const int r = threadIdx.x;
    const bool row_ok = r < H;
    const int rr = row_ok ? r : H - 1;
    const int o_lane = r & 3;
    const unsigned Wst = row_ok ? (unsigned)W : 0u;   // columns this lane may store

    // Element (ch, r, c) of this image, in solve coordinates, sits at
    // chan[ch] (uniform pointer) + rowoff (per lane) +- 4c bytes: one 32-bit lane
    // offset serves all channels, the addressing form global loads take directly.
    const size_t img = (size_t)blockIdx.x * C * H * W;
    const char *chan_src[C];
    char *chan_dst[C];
#pragma unroll
    for (int ch = 0; ch < C; ++ch) {
        const size_t cb = img + (size_t)(DIR ? C - 1 - ch : ch) * H * W;
        chan_src[ch] = reinterpret_cast<const char *>(in + cb);
        chan_dst[ch] = reinterpret_cast<char *>(out + cb);
    }
    constexpr int kStep = DIR ? -4 : 4;               // bytes per column in solve order
    const int row0 = 4 * (DIR ? (H - 1 - rr) * W + (W - 1) : rr * W);   // byte offset of column 0
    const int rowlo = DIR ? row0 - 4 * (W - 1) : row0;                   // lowest / highest byte offset
    const int rowhi = DIR ? row0 : row0 + 4 * (W - 1);                   // inside this row
    auto clamp_row = [&](int off) -> unsigned { return (unsigned)(off < rowlo ? rowlo : (off > rowhi ? rowhi : off)); };
    auto ld = [&](int ch, unsigned off) -> float { return *reinterpret_cast<const float *>(chan_src[ch] + off); };
    auto st = [&](int ch, unsigned off, float v) { *reinterpret_cast<float *>(chan_dst[ch] + off) = v; };

    // Loads are unconditional (offset clamped into the row) so that they stay in
    // flight for kWavePF steps without the compiler having to assume the worst at
    // control-flow joins; out-of-range loads are zeroed when consumed.  Slot s holds
    // the input of the steps congruent to s.  The first batch is issued before the
    // weight preparation so that both latencies overlap.
    float yb[kWavePF][C];
#pragma unroll
    for (int u = 0; u < kWavePF; ++u) {
        const unsigned off = clamp_row(row0 + kStep * (u - r));
#pragma unroll
        for (int ch = 0; ch < C; ++ch)
            yb[u][ch] = ld(ch, off);
    }

    fold_weights<DIR>(w, C, K, sL, sLinv, sCf);
    for (int idx = threadIdx.x; idx < K * K * C * 4; idx += 64) {
        const int o = idx & 3, i = (idx >> 2) % C, tp = idx / (4 * C);
        sA[idx] = (o < C) ? -sCf[(tp * C + o) * C + i] : 0.0f;
    }
    for (int idx = threadIdx.x; idx < C * 4; idx += 64) {
        const int o = idx & 3, j = idx >> 2;
        sLi[idx] = (o < C) ? sLinv[o * C + j] : 0.0f;
    }
    __syncthreads();

    // MFMA A operands (lane holds the entry of output channel o = lane%4, 0 for o >= C):
    // wA[a][db][i] = -Cf[a,db][o][i], wLi[j] = Linv[o][j]
    float wA[K][K][C], wLi[C];
#pragma unroll
    for (int a = 0; a < K; ++a)
#pragma unroll
        for (int db = 0; db < K; ++db)
#pragma unroll
            for (int i = 0; i < C; ++i)
                wA[a][db][i] = sA[((a * K + db) * C + i) * 4 + o_lane];
#pragma unroll
    for (int j = 0; j < C; ++j)
        wLi[j] = sLi[j * 4 + o_lane];

    float xh[C][K];      // xh[i][db] = x(r, c-db), db >= 1
    f32x4 T[K];          // T[a][o], a >= 1: message for pixel (r+a, c), negated sums
#pragma unroll
    for (int i = 0; i < C; ++i) {
#pragma unroll
        for (int db = 0; db < K; ++db)
            xh[i][db] = 0.0f;
    }
#pragma unroll
    for (int a = 0; a < K; ++a)
        T[a] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Have every initial load landed before the loop, so that inside the loop the
    // compiler's wait counts only need to cover the loads of the loop itself.
#pragma unroll
    for (int u = 0; u < kWavePF; ++u)
#pragma unroll
        for (int ch = 0; ch < C; ++ch)
            asm volatile("" : "+v"(yb[u][ch]));

    // own = Linv y - (own-row taps), everything of the coming pixel that does not
    // depend on the rows above; prepared one step ahead.
    int c = -r;                                       // column of this lane at the current step
    int ldoff = row0 + kStep * (kWavePF - r);         // unclamped offset of the next refill
    f32x4 own = f32x4{0.f, 0.f, 0.f, 0.f};
    {
        const bool in_row = (unsigned)c < (unsigned)W;
#pragma unroll
        for (int j = 0; j < C; ++j)
            own = __builtin_amdgcn_mfma_f32_4x4x1f32(wLi[j], in_row ? yb[0][j] : 0.0f, own, 0, 0, 0);
        const unsigned off = clamp_row(ldoff);
#pragma unroll
        for (int ch = 0; ch < C; ++ch)
            yb[0][ch] = ld(ch, off);
        ldoff += kStep;
    }

    const int nsteps = H + W - 1;
    for (int t0 = 0; t0 < nsteps; t0 += kWavePF) {
#pragma unroll
        for (int u = 0; u < kWavePF; ++u) {
            // x(r,c) = own + (message from the row above, computed there one step ago)
            float xn[C];
#pragma unroll
            for (int o = 0; o < C; ++o)
                xn[o] = own[o] + from_lane_above(T[1][o]);
            if ((unsigned)c < Wst) {
                const unsigned off = (unsigned)(row0 + kStep * c);
#pragma unroll
                for (int o = 0; o < C; ++o)
                    st(o, off, xn[o]);
            }
#pragma unroll
            for (int i = 0; i < C; ++i)
                xh[i][0] = xn[i];
            // messages for the rows below: T[a] = S[a+1] + this row's taps
#pragma unroll
            for (int a = 1; a < K; ++a) {
                f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
                if (a + 1 < K) {
#pragma unroll
                    for (int o = 0; o < C; ++o)
                        acc[o] = from_lane_above(T[a + 1][o]);
                }
#pragma unroll
                for (int db = 0; db < K; ++db)
#pragma unroll
                    for (int i = 0; i < C; ++i)
                        acc = __builtin_amdgcn_mfma_f32_4x4x1f32(wA[a][db][i], xh[i][db], acc, 0, 0, 0);
                T[a] = acc;
            }
            // shift the row history and prepare `own` for the next pixel
#pragma unroll
            for (int i = 0; i < C; ++i)
#pragma unroll
                for (int db = K - 1; db >= 1; --db)
                    xh[i][db] = xh[i][db - 1];
            c += 1;
            {
                const int s = (u + 1) % kWavePF;     // slot of the next step (static after unrolling)
                const bool in_row = (unsigned)c < (unsigned)W;
                f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < C; ++j)
                    acc = __builtin_amdgcn_mfma_f32_4x4x1f32(wLi[j], in_row ? yb[s][j] : 0.0f, acc, 0, 0, 0);
#pragma unroll
                for (int db = 1; db < K; ++db)
#pragma unroll
                    for (int i = 0; i < C; ++i)
                        acc = __builtin_amdgcn_mfma_f32_4x4x1f32(wA[0][db][i], xh[i][db], acc, 0, 0, 0);
                own = acc;
                // refill the slot with the input kWavePF steps later
                const unsigned off = clamp_row(ldoff);
#pragma unroll
                for (int ch = 0; ch < C; ++ch)
                    yb[s][ch] = ld(ch, off);
                ldoff += kStep;
            }
        }
    }
}

template <int C, int K>
static int launch_wave_ck(int dir, const float *in, const float *w, float *out, int B, int H, int W,
                          hipStream_t stream)
{
    if (dir)
        hipLaunchKernelGGL((k_solve_wave<C, K, 1>), dim3(B), dim3(64), 0, stream, in, w, out, H, W);
    else
        hipLaunchKernelGGL((k_solve_wave<C, K, 0>), dim3(B), dim3(64), 0, stream, in, w, out, H, W);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

bool wave_supported(int C, int H, int k)
{
    if (H > 64)
        return false;
    return (C == 3 && (k == 3 || k == 5)) || (C == 1 && k == 3) || (C == 2 && k == 3) || (C == 4 && k == 3);
}

int launch_solve_wave(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W, int k,
                      hipStream_t stream)
{
    if (!wave_supported(C, H, k))
        return INVCONV_ERR_VARIANT;
    if (C == 3 && k == 3) return launch_wave_ck<3, 3>(dir, in, w, out, B, H, W, stream);
    if (C == 3 && k == 5) return launch_wave_ck<3, 5>(dir, in, w, out, B, H, W, stream);
    if (C == 1 && k == 3) return launch_wave_ck<1, 3>(dir, in, w, out, B, H, W, stream);
    if (C == 2 && k == 3) return launch_wave_ck<2, 3>(dir, in, w, out, B, H, W, stream);
    if (C == 4 && k == 3) return launch_wave_ck<4, 3>(dir, in, w, out, B, H, W, stream);
    return INVCONV_ERR_VARIANT;
}

}  // namespace invconv
