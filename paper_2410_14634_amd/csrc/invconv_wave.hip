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
#include "invconv_small_mat.h"
#include "invconv_wave_solve.h"
#include <type_traits>
#include <utility>

namespace invconv {

// log|det dx/dy| of one image (Section 4), -H*W*sum_c log|w[c][c][K-1][K-1]|, by the calling wave: the
// forward kernels of few-channel images write it on the side (first workgroup only), so that a training
// step needs no launch of its own for it.  Every lane computes the same value from uniform loads.
template <int C, int K>
__device__ __forceinline__ void wave_logdet(const float *__restrict__ w, int H, int W, float *__restrict__ out)
{
    double s = 0.0;
#pragma unroll
    for (int c = 0; c < C; ++c)
        s += log(fabs((double)w[((c * C + c) * K + (K - 1)) * K + (K - 1)]));
    if ((threadIdx.x & 63) == 0)
        out[0] = (float)(-(double)H * (double)W * s);
}

template <int C, int K, int DIR>
__global__ __launch_bounds__(64) void k_solve_wave(const float *__restrict__ in, const float *__restrict__ w,
                                                  float *__restrict__ out, int H, int W, float *logdet)
{
    if (logdet && blockIdx.x == 0)
        wave_logdet<C, K>(w, H, W, logdet);
    solve_wave_body<C, K, DIR, false>(in, w, out, H, W, blockIdx.x, nullptr);
}

// The same solve on an image held in LDS: the wave copies the image in with 16-byte pieces of
// consecutive lanes, solves in place and copies the result out the same way, so global memory sees
// whole cache lines instead of 64 row-strided 4-byte accesses per instruction (for large batches,
// where those keep more lines live than the L2 holds).  Needs C*H*W a multiple of 4 and 16-byte
// aligned tensors.
// Storage type ST of the activations in memory: float, or bf16 (unsigned short holding the upper half of a
// float; the arithmetic stays fp32, the tile in LDS is float either way).  Four consecutive elements:
typedef unsigned short bf16_t;
__device__ __forceinline__ float bf16_to_float(bf16_t h) { return __builtin_bit_cast(float, (unsigned)h << 16); }
__device__ __forceinline__ bf16_t float_to_bf16(float f)      // round to nearest even; NaN stays NaN
{
    const unsigned u = __builtin_bit_cast(unsigned, f);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (bf16_t)((u >> 16) | 0x40u);
    return (bf16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}
template <typename ST> __device__ __forceinline__ float4 ld4(const ST *base, int i);
template <> __device__ __forceinline__ float4 ld4<float>(const float *base, int i)
{
    return reinterpret_cast<const float4 *>(base)[i];
}
template <> __device__ __forceinline__ float4 ld4<bf16_t>(const bf16_t *base, int i)
{
    const uint2 raw = reinterpret_cast<const uint2 *>(base)[i];
    return make_float4(__builtin_bit_cast(float, raw.x << 16), __builtin_bit_cast(float, raw.x & 0xffff0000u),
                       __builtin_bit_cast(float, raw.y << 16), __builtin_bit_cast(float, raw.y & 0xffff0000u));
}
template <typename ST> __device__ __forceinline__ void st4(ST *base, int i, float4 v);
template <> __device__ __forceinline__ void st4<float>(float *base, int i, float4 v)
{
    reinterpret_cast<float4 *>(base)[i] = v;
}
template <> __device__ __forceinline__ void st4<bf16_t>(bf16_t *base, int i, float4 v)
{
    uint2 raw;
    raw.x = (unsigned)float_to_bf16(v.x) | ((unsigned)float_to_bf16(v.y) << 16);
    raw.y = (unsigned)float_to_bf16(v.z) | ((unsigned)float_to_bf16(v.w) << 16);
    reinterpret_cast<uint2 *>(base)[i] = raw;
}
__device__ __forceinline__ float ld1(const float *p) { return *p; }
__device__ __forceinline__ float ld1(const bf16_t *p) { return bf16_to_float(*p); }

template <int C, int K, int DIR, typename ST = float>
__global__ __launch_bounds__(64) void k_solve_wave_tile(const ST *__restrict__ in, const float *__restrict__ w,
                                                       ST *__restrict__ out, int H, int W, float *logdet)
{
    extern __shared__ float smem[];
    if (logdet && blockIdx.x == 0)
        wave_logdet<C, K>(w, H, W, logdet);
    const int n4 = C * H * W / 4, lane = threadIdx.x;
    const ST *src = in + (size_t)blockIdx.x * C * H * W;
    ST *dst = out + (size_t)blockIdx.x * C * H * W;
    float4 *tile = reinterpret_cast<float4 *>(smem);
    for (int i = lane; i < n4; i += 8 * 64) {
        float4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            v[u] = ld4<ST>(src, i + 64 * u < n4 ? i + 64 * u : n4 - 1);
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (i + 64 * u < n4)
                tile[i + 64 * u] = v[u];
    }
    // (the body works on the LDS tile only; it never touches the global pointers in this mode)
    solve_wave_body<C, K, DIR, false, false, true>(nullptr, w, nullptr, H, W, blockIdx.x, smem);
    for (int i = lane; i < n4; i += 64)
        st4<ST>(dst, i, tile[i]);
}

// Images of at most 32 rows leave half of the wave's lanes idle, and at large batches the solve is bound by
// the instructions a SIMD can issue (27 matrix instructions of 8 clocks per step at C = k = 3, whatever
// the number of rows): here a wave takes two neighbouring images, one per half (solve_wave_body with PACK).
// Lane r of either half reads word r (W - 1) + t of its tile: an odd stride, so the 32 lanes of a half,
// which LDS serves on their own, fall into 32 different banks.  The second tile sits kTilePackPad floats
// behind the end of the first.
// LDS holds few such pairs per compute unit, too few waves to hide the copy in and out behind other
// waves' solves, so a wave hides its own: it walks over pairs (pair = wave index + a multiple of the
// number of waves launched) and fetches the next pair into registers while it solves the current one; after
// the solve each 16-byte piece of the result leaves the tile and the next pair's piece takes its place.
// Pairs of at most 64 * kTile2Pieces pieces (3x32x32 and smaller).  The waves of a workgroup are independent
// (own tile, no barrier); four of them per workgroup put one wave on every SIMD of a compute unit.
constexpr int kTilePackPad = 32;
constexpr int kTile2Pieces = 24;
template <int C, int K, int DIR>
__global__ __launch_bounds__(256) void k_solve_wave_tile2(const float *__restrict__ in, const float *__restrict__ w,
                                                         float *__restrict__ out, int B, int H, int W, float *logdet)
{
    extern __shared__ float smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    if (logdet && blockIdx.x == 0 && wave == 0)
        wave_logdet<C, K>(w, H, W, logdet);
    const int chw = C * H * W, n4 = chw / 4;
    float *slot = smem + wave * (2 * chw + kTilePackPad);
    float4 *tile = reinterpret_cast<float4 *>(slot);
    const int npairs = (B + 1) >> 1, stride = gridDim.x * nw;
    auto pieces_of = [&](int q) { return 2 * q + 1 < B ? 2 * n4 : n4; };      // the last pair may be a single image
    auto at = [&](int i) { return i < n4 ? i : i + kTilePackPad / 4; };
    int p = blockIdx.x * nw + wave;
    if (p >= npairs)
        return;
    float4 v[kTile2Pieces];
    auto fetch = [&](int q) {
        const float *src = in + (size_t)2 * q * chw;
        const int t4 = pieces_of(q);
#pragma unroll
        for (int u = 0; u < kTile2Pieces; ++u)
            v[u] = ld4<float>(src, lane + 64 * u < t4 ? lane + 64 * u : t4 - 1);
    };
    fetch(p);
    {
        const int t4 = pieces_of(p);
#pragma unroll
        for (int u = 0; u < kTile2Pieces; ++u)
            if (lane + 64 * u < t4)
                tile[at(lane + 64 * u)] = v[u];
    }
    for (;;) {
        const int pn = p + stride;
        const bool more = pn < npairs;
        if (more)
            fetch(pn);
        solve_wave_body<C, K, DIR, false, false, true, true>(nullptr, w, nullptr, H, W, 0, slot, WaveBands{},
                                                             2 * p + 1 < B, chw + kTilePackPad);
        float *dst = out + (size_t)2 * p * chw;
        const int tc = pieces_of(p), tn = more ? pieces_of(pn) : 0;
#pragma unroll
        for (int u = 0; u < kTile2Pieces; ++u) {
            const int i = lane + 64 * u;
            if (i < tc)
                st4<float>(dst, i, tile[at(i)]);
            if (i < tn)
                tile[at(i)] = v[u];
        }
        if (!more)
            break;
        p = pn;
    }
}

// ---------------------------------------------------------------------------
// The same solve with the matrix instructions of a step split over the waves of a workgroup by the age of
// their input (images of at most 64 rows; pays when a step is long; four waves up to k = 5, k/2 + 2.5 waves
// beyond).  With
// x_s the diagonal solved at step s and A[a][db] the folded taps (lane = row, as above),
//   T[a]_s    = up(T[a+1]_{s-1}) + A[a][0] x_s + { sum_{db>=1} A[a][db] x_{s-db} }   = Tp[a]_s + F[a]_s
//   own_{s+1} =                    A[0][1] x_s + { Linv y_{s+1} + sum_{db>=2} A[0][db] x_{s+1-db} }
//                                                                                    = ownp_s + O_{s+1}
//   x_{s+1}   = own_{s+1} + up(T[1]_s)
// The braces need nothing newer than x_{s-1}.  Wave 0, on the chain of dependent steps, publishes x_s
// through LDS and forms Tp and ownp (K*C instructions); during step s waves 1 .. NF form the F[a]_s, the
// last wave forms O_{s+1}, reads y and writes x_{s-1} to global memory; wave 0 picks the results up
// after the barrier that ends the step.  Every wave runs its own loop over the same number of steps.
// ---------------------------------------------------------------------------
struct WaveSplitLds {
    float *x;       // [2][C][64]   x of the last two steps
    f32x4 *m;       // [2][K][64]   slot 0: O, slot a: F[a]
};

template <int C, int K>
__host__ __device__ constexpr size_t wave_split_lds_floats() { return 2 * C * 64 + 2 * K * 64 * 4; }

// NF waves share the F[a] (wave f = 1 .. NF takes (K-1)/NF consecutive a; two waves for k <= 5, one per two a
// from k = 7 on, so that no wave has more than 2 (K-1) C matrix instructions in a step); wave NF + 1 forms O.
// Every role folds the weights for itself after the set-up barrier, so that only the taps it uses stay in
// registers (all C K K folded taps of k = 11 are more than a wave of a large workgroup may hold).
__host__ __device__ constexpr int wave_split_nf(int K) { return K >= 7 ? (K - 1) / 2 : 2; }

template <class F, int... Is>
__device__ __forceinline__ void wave_split_dispatch(int wave, F &&f, std::integer_sequence<int, Is...>)
{
    ((wave == Is + 1 ? (f(std::integral_constant<int, Is>{}), 0) : 0), ...);
}

// The neighbours of the inverse convolution in a flow step (Section 4.1: Actnorm a = s x + b, then the 1 x 1
// convolution z = Q a) as the kernels of few channels take them: the three parameter tensors in memory; a wave
// that needs the channel map z = A x + d (A = Q diag(s), d = Q b) forms it in registers.
struct FlowParams {
    const float *s, *b, *Q;
};

template <int C>
__device__ __forceinline__ void flow_map_regs(FlowParams fp, float (&A)[C][C], float (&d)[C])
{
#pragma unroll
    for (int o = 0; o < C; ++o) {
        double acc = 0.0;
#pragma unroll
        for (int i = 0; i < C; ++i) {
            A[o][i] = fp.Q[o * C + i] * fp.s[i];
            acc += (double)fp.Q[o * C + i] * (double)fp.b[i];
        }
        d[o] = (float)acc;
    }
}

// log|det dz/dy| of one image for the whole step, by one wave (every lane the same arithmetic, lane 0 writes):
//   H W ( sum log|s[c]| + log|det Q| - sum log|w[c][c][k-1][k-1]| )        (Section 4)
template <int C, int K>
__device__ __forceinline__ void flow_logdet_small(const float *__restrict__ w, FlowParams fp, int H, int W,
                                                  float *__restrict__ out)
{
    double q[C][C], qi[C][C];
#pragma unroll
    for (int o = 0; o < C; ++o)
#pragma unroll
        for (int i = 0; i < C; ++i)
            q[o][i] = (double)fp.Q[o * C + i];
    double acc = log(fabs(small_det_inv<C>(q, qi)));
#pragma unroll
    for (int c = 0; c < C; ++c)
        acc += log(fabs((double)fp.s[c])) - log(fabs((double)w[((c * C + c) * K + (K - 1)) * K + (K - 1)]));
    if ((threadIdx.x & 63) == 0)
        out[0] = (float)((double)H * (double)W * acc);
}

// MAP, forward direction: the wave that stores x applies the flow step's channel map on the way out, so what
// reaches memory is z = A x + d; x stays in the workgroup.  MAP, transposed direction: the input is dL/dz and the
// solve wants A^T dL/dz; the input enters only through Linv y, so A^T is folded into Linv once (in mirrored channel
// order, like everything else in that direction).
template <int C, int K, int DIR, bool LDS_COPY, int NF = 2, bool MAP = false>
__device__ __forceinline__ void solve_wave_split_body(const float *__restrict__ in, const float *__restrict__ w,
                                                      float *__restrict__ out, int H, int W, int n, float *lds_copy,
                                                      WaveSplitLds sl, FlowParams fp = FlowParams{})
{
    static_assert(C >= 1 && C <= 4 && K >= 3, "one 4-row MFMA block per pixel");
    static_assert(!MAP || DIR == 1 || !LDS_COPY, "the outgoing channel map goes with the plain forward solve");
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane;
    const bool row_ok = r < H;
    const int rr = row_ok ? r : H - 1;
    const int o_lane = r & 3;
    const unsigned Wst = row_ok ? (unsigned)W : 0u;

    const size_t img = (size_t)n * C * H * W;
    const char *chan_src[C];
    char *chan_dst[C];
    char *chan_lds[C];
#pragma unroll
    for (int ch = 0; ch < C; ++ch) {
        const size_t cb = (size_t)(DIR ? C - 1 - ch : ch) * H * W;
        chan_src[ch] = reinterpret_cast<const char *>(in + img + cb);
        chan_dst[ch] = reinterpret_cast<char *>(out + img + cb);
        chan_lds[ch] = reinterpret_cast<char *>(lds_copy + cb);
    }
    constexpr int kStep = DIR ? -4 : 4;
    const int row0 = 4 * (DIR ? (H - 1 - rr) * W + (W - 1) : rr * W);
    const int rowlo = DIR ? row0 - 4 * (W - 1) : row0;
    const int rowhi = DIR ? row0 : row0 + 4 * (W - 1);
    auto clamp_row = [&](int off) -> unsigned { return (unsigned)(off < rowlo ? rowlo : (off > rowhi ? rowhi : off)); };

    // the last wave reads y: slot u holds the input of the steps congruent to u.  The other waves run the same
    // instructions on one common address (no branch around a load, next to no work for the address unit).
    constexpr int kOWave = NF + 1;
    float yb[kWavePF][C];
#pragma unroll
    for (int u = 0; u < kWavePF; ++u) {
        const unsigned off = wave == kOWave ? clamp_row(row0 + kStep * (u - r)) : 0u;
#pragma unroll
        for (int ch = 0; ch < C; ++ch)
            yb[u][ch] = *reinterpret_cast<const float *>((wave == kOWave ? chan_src[ch] : chan_src[0]) + off);
    }

    for (int idx = threadIdx.x; idx < (int)wave_split_lds_floats<C, K>(); idx += 64 * (NF + 2))
        sl.x[idx] = 0.0f;       // x and message slots are contiguous
#pragma unroll
    for (int u = 0; u < kWavePF; ++u)
#pragma unroll
        for (int ch = 0; ch < C; ++ch)
            asm volatile("" : "+v"(yb[u][ch]));
    __syncthreads();

    // step s = -1 only lets the last wave prepare O_0 = Linv y_0; the steps after the last diagonal only let it store
    const int nsteps = H + W - 1;
    const int total = nsteps + 2;       // steps -1 .. total-2, the same for every wave
    if (wave == 0) {
        float wA[K][K][C], wLi[C];
        wave_fold_regs<C, K, DIR>(w, o_lane, wA, wLi);
        f32x4 Tp[K], ownp = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int a = 0; a < K; ++a)
            Tp[a] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int s = -1; s < total - 1; ++s) {
            // The F[a] arrive already shifted by one lane (their waves have the time for it), so
            // up(T[a]) = up(Tp[a]) + up(F[a]) is one add whose first operand takes the lane shift along.
            const f32x4 *mi = sl.m + ((s - 1) & 1) * K * 64 + lane;
            f32x4 Fs[K];
#pragma unroll
            for (int a = 1; a < K; ++a)
                Fs[a] = mi[a * 64];
            const f32x4 own = ownp + mi[0];
            float xn[C];
#pragma unroll
            for (int o = 0; o < C; ++o) {
                xn[o] = own[o] + (from_lane_above(Tp[1][o]) + Fs[1][o]);
                sl.x[((s & 1) * C + o) * 64 + lane] = xn[o];
            }
#pragma unroll
            for (int a = 1; a < K; ++a) {
                f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
                if (a + 1 < K) {
#pragma unroll
                    for (int o = 0; o < C; ++o)
                        acc[o] = from_lane_above(Tp[a + 1][o]) + Fs[a + 1][o];
                }
#pragma unroll
                for (int i = 0; i < C; ++i)
                    acc = __builtin_amdgcn_mfma_f32_4x4x1f32(wA[a][0][i], xn[i], acc, 0, 0, 0);
                Tp[a] = acc;
            }
            {
                f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int i = 0; i < C; ++i)
                    acc = __builtin_amdgcn_mfma_f32_4x4x1f32(wA[0][1][i], xn[i], acc, 0, 0, 0);
                ownp = acc;
            }
            __syncthreads();
        }
    } else if (wave <= NF) {
        // F[a]_s = sum_{db>=1} A[a][db] x_{s-db} for the wave's own a (fixed at compile time per wave)
        constexpr int PER = (K - 1 + NF - 1) / NF;
        auto f_loop = [&](auto tag) {
            constexpr int A_LO = decltype(tag)::value * PER + 1;
            float wA[K][K][C], wLi[C];
            wave_fold_regs<C, K, DIR>(w, o_lane, wA, wLi);
            float xo[K][C];     // xo[db] = x_{s-db}, db >= 1
#pragma unroll
            for (int db = 0; db < K; ++db)
#pragma unroll
                for (int i = 0; i < C; ++i)
                    xo[db][i] = 0.0f;
            for (int s = -1; s < total - 1; ++s) {
#pragma unroll
                for (int db = K - 1; db >= 2; --db)
#pragma unroll
                    for (int i = 0; i < C; ++i)
                        xo[db][i] = xo[db - 1][i];
#pragma unroll
                for (int i = 0; i < C; ++i)
                    xo[1][i] = sl.x[(((s - 1) & 1) * C + i) * 64 + lane];
                f32x4 *mo = sl.m + (s & 1) * K * 64 + lane;
#pragma unroll
                for (int a = A_LO; a < A_LO + PER; ++a) {
                    if (a >= K)
                        continue;
                    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int db = K - 1; db >= 1; --db)
#pragma unroll
                        for (int i = 0; i < C; ++i)
                            acc = __builtin_amdgcn_mfma_f32_4x4x1f32(wA[a][db][i], xo[db][i], acc, 0, 0, 0);
                    f32x4 up = f32x4{0.f, 0.f, 0.f, 0.f};      // what the row below will add: F[a] of the lane above
#pragma unroll
                    for (int o = 0; o < C; ++o)
                        up[o] = from_lane_above(acc[o]);
                    mo[a * 64] = up;
                }
                __syncthreads();
            }
        };
        wave_split_dispatch(wave, f_loop, std::make_integer_sequence<int, NF>{});
    } else {
        // O_{s+1} = Linv y_{s+1} + sum_{db>=2} A[0][db] x_{s+1-db}; also x_{s-1} to global memory
        float wA[K][K][C], wLi[C];
        wave_fold_regs<C, K, DIR>(w, o_lane, wA, wLi);
        float mA[MAP ? C : 1][MAP ? C : 1], md[MAP ? C : 1];
        if constexpr (MAP) {
            flow_map_regs<C>(fp, mA, md);
            if constexpr (DIR == 1) {
                float folded[C];
#pragma unroll
                for (int j = 0; j < C; ++j) {
                    folded[j] = 0.0f;
#pragma unroll
                    for (int m = 0; m < C; ++m)
                        folded[j] += wLi[m] * mA[C - 1 - j][C - 1 - m];     // (A^T in mirrored order)[m][j]
                }
#pragma unroll
                for (int j = 0; j < C; ++j)
                    wLi[j] = folded[j];
            }
        }
        float xo[K][C];     // xo[db] = x_{s+1-db}, db >= 2
#pragma unroll
        for (int db = 0; db < K; ++db)
#pragma unroll
            for (int i = 0; i < C; ++i)
                xo[db][i] = 0.0f;
        int ldoff = row0 + kStep * (kWavePF - r);       // unclamped offset of the next refill
        // one step; u = slot of the input of step s + 1 (s + 1 is congruent to u)
        auto step = [&](int s, int u, bool refill) {
#pragma unroll
            for (int db = K - 1; db >= 3; --db)
#pragma unroll
                for (int i = 0; i < C; ++i)
                    xo[db][i] = xo[db - 1][i];
#pragma unroll
            for (int i = 0; i < C; ++i)
                xo[2][i] = sl.x[(((s - 1) & 1) * C + i) * 64 + lane];
            const bool in_row = (unsigned)(s + 1 - r) < (unsigned)W;
            f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < C; ++j)
                acc = __builtin_amdgcn_mfma_f32_4x4x1f32(wLi[j], in_row ? yb[u][j] : 0.0f, acc, 0, 0, 0);
#pragma unroll
            for (int db = K - 1; db >= 2; --db)
#pragma unroll
                for (int i = 0; i < C; ++i)
                    acc = __builtin_amdgcn_mfma_f32_4x4x1f32(wA[0][db][i], xo[db][i], acc, 0, 0, 0);
            sl.m[(s & 1) * K * 64 + lane] = acc;
            const int c = s - 1 - r;        // column of x_{s-1} = xo[2] in this lane's row
            if ((unsigned)c < Wst) {
                const unsigned off = (unsigned)(row0 + kStep * c);
#pragma unroll
                for (int o = 0; o < C; ++o) {
                    float val = xo[2][o];
                    if constexpr (MAP && DIR == 0) {
                        val = md[o];
#pragma unroll
                        for (int i = 0; i < C; ++i)
                            val += mA[o][i] * xo[2][i];
                    }
                    *reinterpret_cast<float *>(chan_dst[o] + off) = val;
                    if (LDS_COPY)
                        *reinterpret_cast<float *>(chan_lds[o] + off) = xo[2][o];
                }
            }
            if (refill) {       // the input of step s + 1 + kWavePF
                const unsigned off = clamp_row(ldoff);
#pragma unroll
                for (int ch = 0; ch < C; ++ch)
                    yb[u][ch] = *reinterpret_cast<const float *>(chan_src[ch] + off);
                ldoff += kStep;
            }
            __syncthreads();
        };
        // whole blocks of kWavePF steps, then the rest without refills (its inputs are already there)
        const int nfull = total / kWavePF;
        int s0 = -1;
        for (int blk = 0; blk < nfull; ++blk, s0 += kWavePF) {
#pragma unroll
            for (int u = 0; u < kWavePF; ++u)
                step(s0 + u, u, true);
        }
        const int rest = total - nfull * kWavePF;
#pragma unroll
        for (int u = 0; u < kWavePF; ++u)
            if (u < rest)
                step(s0 + u, u, false);
    }
}

template <int C, int K, int DIR>
__global__ __launch_bounds__(64 * (wave_split_nf(K) + 2)) void k_solve_wave_split(const float *__restrict__ in,
                                                                                  const float *__restrict__ w,
                                                                                  float *__restrict__ out, int H,
                                                                                  int W, float *logdet)
{
    __shared__ __attribute__((aligned(16))) float smem[wave_split_lds_floats<C, K>()];
    if (logdet && blockIdx.x == 0 && (threadIdx.x >> 6) == 1)      // wave 1 has the least to set up
        wave_logdet<C, K>(w, H, W, logdet);
    WaveSplitLds sl;
    sl.x = smem;
    sl.m = reinterpret_cast<f32x4 *>(smem + 2 * C * 64);
    solve_wave_split_body<C, K, DIR, false, wave_split_nf(K)>(in, w, out, H, W, blockIdx.x, nullptr, sl);
}

// Forward pass of a whole flow step for few channels and few images: the split solve with the channel map on its
// way out (y in, z out) and the step's log-determinant on the side; no set-up launch.
template <int C, int K>
__global__ __launch_bounds__(64 * (wave_split_nf(K) + 2)) void k_flow_fwd_split(const float *__restrict__ y,
                                                                                const float *__restrict__ w,
                                                                                FlowParams fp, float *__restrict__ z,
                                                                                int H, int W, float *logdet)
{
    __shared__ __attribute__((aligned(16))) float smem[wave_split_lds_floats<C, K>()];
    if (logdet && blockIdx.x == 0 && (threadIdx.x >> 6) == 1)
        flow_logdet_small<C, K>(w, fp, H, W, logdet);
    WaveSplitLds sl;
    sl.x = smem;
    sl.m = reinterpret_cast<f32x4 *>(smem + 2 * C * 64);
    solve_wave_split_body<C, K, 0, false, wave_split_nf(K), true>(y, w, z, H, W, blockIdx.x, nullptr, sl, fp);
}

// Images of 65 .. 512 rows: one workgroup per image, one wave per band of 64 rows.
template <int C, int K, int DIR>
__global__ __launch_bounds__(512) void k_solve_wave_bands(const float *__restrict__ in, const float *__restrict__ w,
                                                         float *__restrict__ out, int H, int W, int log_steps,
                                                         int spin_limit, int *err)
{
    extern __shared__ float smem[];
    WaveBands wb;
    wb.spin_limit = spin_limit;
    wb.err = err;
    wb.band = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    wb.nbands = blockDim.x >> 6;
    f32x4 *log = reinterpret_cast<f32x4 *>(smem);        // [nbands - 1][log_steps][K - 1]
    wb.scratch = log + (size_t)(wb.nbands - 1) * log_steps * (K - 1);
    int *prog = reinterpret_cast<int *>(wb.scratch + 64 * (K - 1));     // [nbands - 1]
    // (plain offsets from the LDS base, never a null alternative: the accesses stay LDS instructions)
    wb.log_in = log + (size_t)(wb.band > 0 ? wb.band - 1 : 0) * log_steps * (K - 1);
    wb.log_out = log + (size_t)(wb.band + 1 < wb.nbands ? wb.band : 0) * log_steps * (K - 1);
    wb.prog_in = prog + (wb.band > 0 ? wb.band - 1 : 0);
    wb.prog_out = prog + (wb.band + 1 < wb.nbands ? wb.band : 0);
    wb.log_steps = log_steps;
    if (threadIdx.x < wb.nbands - 1)
        prog[threadIdx.x] = 0;
    __syncthreads();
    solve_wave_body<C, K, DIR, false, true>(in, w, out, H, W, blockIdx.x, nullptr, wb);
}

// The courier of a band's workgroup (one wave): carries the two logs between the workgroup's LDS and the
// logs in global memory, a block of kWavePF entries at a time.
template <int K>
__device__ __forceinline__ void bands_courier(f32x4 *log, int *prog, size_t seg, int band, int nb, int n,
                                              int log_steps, int *gcount, f32x4 *glog, int spin_limit, int *err)
{
    const int lane = threadIdx.x & 63;
    const int per_blk = kWavePF * (K - 1);               // 16-byte entries per block (at most 64: K <= 5)
    const int send_total = band + 1 < nb ? log_steps : 0, recv_total = band > 0 ? log_steps : 0;
    int *cnt_out = gcount + (size_t)n * (nb - 1) + (band + 1 < nb ? band : 0);
    const int *cnt_in = gcount + (size_t)n * (nb - 1) + (band > 0 ? band - 1 : 0);
    f32x4 *g_out = glog + ((size_t)n * (nb - 1) + (band + 1 < nb ? band : 0)) * seg;
    const f32x4 *g_in = glog + ((size_t)n * (nb - 1) + (band > 0 ? band - 1 : 0)) * seg;
    const unsigned seg_bytes = (unsigned)(seg * sizeof(f32x4));
    const __amdgpu_buffer_rsrc_t r_out =
        __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void *>(g_out), 0, (int)seg_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t r_in = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void *>(reinterpret_cast<const void *>(g_in)), 0, (int)seg_bytes, 0x00020000);
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    int sent = 0, got = 0, spins = 0;
    while ((sent < send_total || got < recv_total) && spins < spin_limit) {
        bool moved = false;
        if (sent < send_total) {
            int have = __hip_atomic_load(prog + 1, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP);
            have = have < send_total ? have : send_total;
            if (sent < have) {
                while (sent < have) {
                    if (lane < per_blk) {
                        const f32x4 e = log[seg + (size_t)sent * (K - 1) + lane];
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, e), r_out,
                                                               (sent * (K - 1) + lane) * 16, 0, 16 /* sc1 */);
                    }
                    sent += kWavePF;
                }
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_waitcnt(0);          // every store above is acknowledged
                asm volatile("" ::: "memory");
                if (lane == 0)
                    __hip_atomic_store(cnt_out, sent, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                moved = true;
            }
        }
        if (got < recv_total) {
            int avail = __hip_atomic_load(cnt_in, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            avail = avail < recv_total ? avail : recv_total;
            asm volatile("" ::: "memory");              // the loads below are issued after the counter was read
            if (got < avail) {
                while (got < avail) {
                    if (lane < per_blk) {
                        const u32x4 e = __builtin_amdgcn_raw_buffer_load_b128(r_in, (got * (K - 1) + lane) * 16, 0,
                                                                              16 /* sc1 */);
                        log[(size_t)got * (K - 1) + lane] = __builtin_bit_cast(f32x4, e);
                    }
                    got += kWavePF;
                }
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_waitcnt(0);          // the entries are in LDS
                asm volatile("" ::: "memory");
                if (lane == 0)
                    __hip_atomic_store(prog, got, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
                moved = true;
            }
        }
        if (!moved) {
            __builtin_amdgcn_s_sleep(2);
            ++spins;
        }
    }
    // gave up with entries still to carry: the solving waves that depend on them run out of their own
    // waits and store NaN; the error word tells the caller
    if ((sent < send_total || got < recv_total) && err && lane == 0)
        __hip_atomic_store(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The same bands on different compute units: one workgroup per (band, image), two waves each.  Wave 0 is
// the band's solve exactly as above, with its two logs in the workgroup's own LDS.  Wave 1 carries the
// logs between workgroups through global memory, a block of kWavePF entries at a time: it sends what its
// own band has appended (device-coherent stores, then a counter once they are acknowledged - it has no
// other memory operations in flight, so that wait is exact) and fetches what the band above has published
// into the local log, then advances the local counter the solve waits on.  A workgroup waits only for the
// one of the band above, which has a lower block index; every wait is bounded.
template <int C, int K, int DIR>
__global__ __launch_bounds__(128) void k_solve_wave_bands_multi(const float *__restrict__ in,
                                                               const float *__restrict__ w, float *__restrict__ out,
                                                               int B, int H, int W, int log_steps, int *gcount,
                                                               f32x4 *glog, int spin_limit, int *err)
{
    extern __shared__ float smem[];
    const int nb = (H + 63) >> 6;
    const int band = blockIdx.x / B, n = blockIdx.x % B;
    const size_t seg = (size_t)log_steps * (K - 1);
    f32x4 *log = reinterpret_cast<f32x4 *>(smem);        // [2][log_steps][K - 1]: received, sent
    f32x4 *scratch = log + 2 * seg;
    int *prog = reinterpret_cast<int *>(scratch + 64 * (K - 1));        // [2]: received, sent
    if (threadIdx.x < 2)
        prog[threadIdx.x] = 0;
    __syncthreads();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (wave == 0) {
        WaveBands wb;
        wb.band = band;
        wb.nbands = nb;
        wb.log_in = log;
        wb.log_out = log + seg;
        wb.prog_in = prog;
        wb.prog_out = prog + 1;
        wb.log_steps = log_steps;
        wb.scratch = scratch;
        wb.spin_limit = spin_limit;
        wb.err = err;
        solve_wave_body<C, K, DIR, false, true>(in, w, out, H, W, n, nullptr, wb);
        return;
    }
    bands_courier<K>(log, prog, seg, band, nb, n, log_steps, gcount, glog, spin_limit, err);
}

__global__ void k_wave_bands_clear(int *gcount, int count)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count)
        gcount[i] = 0;
}

// ---------------------------------------------------------------------------
// Bands on different compute units with whole-line memory traffic (W a multiple of 4): four waves per
// (band, image).  Wave 0 solves as above but reads its input from, and writes its result into, an LDS
// ring of kRingCols columns per row (in place); wave 1 is the courier of the logs; wave 2 fills the ring
// and wave 3 drains it, both with 16-byte accesses of which four neighbouring lanes cover 64 contiguous
// bytes of one row.  The solving wave itself then issues no memory instruction whose lanes touch 64
// different cache lines, which is what bounds the step of the kernel above.
//
// Schedule, in blocks of kWavePF steps and chunks of kWavePF columns (rho(r) = floor((r-1)/16)):
//   load block m    row r receives chunk m - rho(r), m = -1, 0, ...; the solve starts block j once load blocks
//                   <= j are in LDS;
//   solve block j   row r reads chunks j - rho - 1 and j - rho and overwrites columns 16j - r .. 16j+15 - r;
//   store block m   after solve block m, row r's chunk m - rho - 1 is complete and leaves.
// A slot is therefore held by chunk q of row r from load block q + rho to store block q + rho + 1, and the
// chunk q + 4 that takes the same slot is written by load block q + rho + 4, which waits until store block
// q + rho + 1 has read the slot.  The filling wave keeps the loads of the next two blocks in flight in its
// registers, so the wait for a slot does not expose memory latency.  Dependencies only point to earlier
// blocks, every wait is bounded, and a wave that gives up sets the error word and passes NaN on.
// ---------------------------------------------------------------------------
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bool wait_count(const int *counter, int need, int spin_limit)
{
    int spins = 0;
    while (__hip_atomic_load(counter, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < need && ++spins < spin_limit)
        __builtin_amdgcn_s_sleep(1);
    return __hip_atomic_load(counter, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) >= need;
}

// Byte offset of the four columns 16q + 4p .. + 3 (solve coordinates) of band row `row`, channel ch, inside
// the image, or an offset past the image (the buffer unit then returns zeros / drops the store).
template <int C, int DIR>
__device__ __forceinline__ unsigned ring_item_offset(int ch, int row, int q, int p, int band, int band_rows, int H,
                                                     int W, bool need_row)
{
    const int cs0 = 16 * q + 4 * p;
    const bool ok = q >= 0 && cs0 < W && (!need_row || row < band_rows);
    const int rc = row < band_rows ? row : band_rows - 1;
    const int grow = 64 * band + rc;
    const int mrow = DIR ? H - 1 - grow : grow, mcol = DIR ? W - 4 - cs0 : cs0, mch = DIR ? C - 1 - ch : ch;
    return ok ? (unsigned)((((size_t)mch * H + mrow) * W + mcol) * sizeof(float)) : 0x80000000u;
}

template <int C, int K, int DIR>
__global__ __launch_bounds__(256) void k_solve_wave_bands_io(const float *__restrict__ in, const float *__restrict__ w,
                                                            float *__restrict__ out, int B, int H, int W,
                                                            int log_steps, int *gcount, f32x4 *glog, int spin_limit,
                                                            int spin_courier, int *err)
{
    extern __shared__ float smem[];
    const int nb = (H + 63) >> 6;
    const int band = blockIdx.x / B, n = blockIdx.x % B;
    const size_t seg = (size_t)log_steps * (K - 1);
    f32x4 *log = reinterpret_cast<f32x4 *>(smem);        // [2][log_steps][K - 1]: received, sent
    f32x4 *scratch = log + 2 * seg;
    float *ring = reinterpret_cast<float *>(scratch + 64 * (K - 1));    // [C][64][kRingStride]
    int *prog = reinterpret_cast<int *>(ring + C * 64 * kRingStride);    // received, sent, loaded, done, stored, lost
    if (threadIdx.x < 6)
        prog[threadIdx.x] = (threadIdx.x == 0 && band == 0) ? log_steps : 0;
    if (band == 0) {    // nothing comes from above the first band: its incoming log is zeros, already complete
        for (int i = threadIdx.x; i < (int)seg; i += 256)
            log[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    __syncthreads();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int band_rows = H - 64 * band < 64 ? H - 64 * band : 64;
    const int nblocks = (band_rows + W - 1 + kWavePF - 1) / kWavePF;     // blocks of the solve
    int *io_loaded = prog + 2, *io_done = prog + 3, *io_stored = prog + 4, *io_lost = prog + 5;
    if (wave == 0) {
        WaveBands wb;
        wb.band = band;
        wb.nbands = nb;
        wb.log_in = log;
        wb.log_out = log + seg;
        wb.prog_in = prog;
        wb.prog_out = prog + 1;
        wb.log_steps = log_steps;
        wb.scratch = scratch;
        wb.spin_limit = spin_limit;
        wb.err = err;
        wb.ring = ring;
        wb.io_loaded = io_loaded;
        wb.io_done = io_done;
        wb.io_lost = io_lost;
        solve_wave_ring_body<C, K, DIR>(w, H, W, wb);
        return;
    }
    if (wave == 1) {
        bands_courier<K>(log, prog, seg, band, nb, n, log_steps, gcount, glog, spin_courier, err);
        return;
    }
    const int lane = threadIdx.x & 63, p = lane & 3, rsub = lane >> 2;
    const size_t img = (size_t)n * C * H * W;
    const int img_bytes = (int)((size_t)C * H * W * sizeof(float));
    if (wave == 2) {
        // ---- fills the ring
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<void *>(reinterpret_cast<const void *>(in + img)), 0, img_bytes, 0x00020000);
        bool lost = false;
        u32x4_t s0[4 * C], s1[4 * C], s2[4 * C];
        auto issue = [&](int m, u32x4_t(&regs)[4 * C]) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = 16 * i + rsub, q = m - ring_rho(row);
#pragma unroll
                for (int ch = 0; ch < C; ++ch)
                    regs[i * C + ch] = __builtin_amdgcn_raw_buffer_load_b128(
                        rs, ring_item_offset<C, DIR>(ch, row, q, p, band, band_rows, H, W, false), 0, 0);
            }
        };
        auto land = [&](int m, u32x4_t(&regs)[4 * C]) {
            if (m >= nblocks)
                return;
            // the slots of this block were last read by store block m - 3
            if (!lost && m >= 3 && !wait_count(io_stored, m - 2, spin_limit)) {
                lost = true;
                __hip_atomic_store(io_lost, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                if (err && lane == 0)
                    __hip_atomic_store(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = 16 * i + rsub, q = m - ring_rho(row), cs0 = 16 * q + 4 * p;
                if (q >= 0 && cs0 < W) {
#pragma unroll
                    for (int ch = 0; ch < C; ++ch) {
                        f32x4 v = __builtin_bit_cast(f32x4, regs[i * C + ch]);
                        if (DIR)
                            v = f32x4{v[3], v[2], v[1], v[0]};
                        if (lost)
                            v = f32x4{__builtin_nanf(""), __builtin_nanf(""), __builtin_nanf(""), __builtin_nanf("")};
                        *reinterpret_cast<f32x4 *>(ring + (ch * 64 + row) * kRingStride + (cs0 & (kRingCols - 1))) = v;
                    }
                }
            }
            __hip_atomic_store(io_loaded, m + 2, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        };
        // blocks -1 .. nblocks - 1 (block -1 carries the first chunk of row 0, whose rho is -1)
        issue(-1, s0);
        issue(0, s1);
        for (int m = -1; m < nblocks; m += 3) {
            issue(m + 2, s2);
            land(m, s0);
            issue(m + 3, s0);
            land(m + 1, s1);
            issue(m + 4, s1);
            land(m + 2, s2);
        }
        return;
    }
    // ---- drains the ring
    const __amdgpu_buffer_rsrc_t rd =
        __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void *>(out + img), 0, img_bytes, 0x00020000);
    bool lost = false;
    const int nstore = (W + 15) / 16 + 4;      // the last chunk of the last row leaves with store block W/16 + 3
    for (int m = 0; m < nstore; ++m) {
        const int need = m + 1 < nblocks ? m + 1 : nblocks;
        if (!lost && !wait_count(io_done, need, spin_limit)) {
            lost = true;
            if (err && lane == 0)
                __hip_atomic_store(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        f32x4 v[4 * C];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = 16 * i + rsub, q = m - ring_rho(row) - 1, cs0 = 16 * q + 4 * p;
#pragma unroll
            for (int ch = 0; ch < C; ++ch)
                v[i * C + ch] =
                    *reinterpret_cast<const f32x4 *>(ring + (ch * 64 + row) * kRingStride + (cs0 & (kRingCols - 1)));
        }
        // a wave that ran on after a lost wait no longer keeps to the schedule of the ring: nothing read from
        // now on is known to be a result (the flag was set before the counter that let this block through)
        lost = lost || __hip_atomic_load(io_lost, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) != 0;
        // (the release waits for the reads above to have returned)
        __hip_atomic_store(io_stored, m + 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = 16 * i + rsub, q = m - ring_rho(row) - 1;
#pragma unroll
            for (int ch = 0; ch < C; ++ch) {
                f32x4 e = v[i * C + ch];
                if (DIR)
                    e = f32x4{e[3], e[2], e[1], e[0]};
                if (lost)
                    e = f32x4{__builtin_nanf(""), __builtin_nanf(""), __builtin_nanf(""), __builtin_nanf("")};
                __builtin_amdgcn_raw_buffer_store_b128(
                    __builtin_bit_cast(u32x4_t, e), rd,
                    ring_item_offset<C, DIR>(ch, row, q, p, band, band_rows, H, W, true), 0, 0);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Backward pass of one image in one workgroup of four waves (Section 3.1-3.3).
//   wave 0      transposed solve v = dL/dy (mirrored orientation), written to
//               global memory and to an LDS tile;
//   waves 1..3  meanwhile stage the image's x, with a zero halo of K-1 rows and
//               columns on the top/left, in LDS;
//   all waves   then form the image's share of the weight gradient (Eq. 4 with
//               Theorem 2), sum_p v[o][p] * x[i][p - tap], as outer products on the
//               matrix cores: v_mfma_f32_4x4x1 has 16 independent 4x4 blocks, block b
//               takes pixel 16q+b, its A operand is v[o = lane%4] of that pixel and
//               its B operand four of the C*K*K shifted-x columns.  The 16 block
//               accumulators of the four waves are added in a fixed order through LDS.
// Output: part[n][P] un-negated; a second kernel adds the images in index order.
// ---------------------------------------------------------------------------
// With SPLIT all four waves stage x first and then run the transposed solve with its steps split over
// the waves (solve_wave_split_body); its exchange buffers sit behind the tiles.
// With TILE (large batches, see wave_tile_preferred) all four waves first bring dL/dx and x into LDS with
// accesses of consecutive lanes, wave 0 solves in place in LDS, and dL/dy leaves the same way afterwards.
template <int C, int K, bool SPLIT, bool TILE = false, typename ST = float>
__global__ __launch_bounds__(256) void k_bwd_wave(const ST *__restrict__ x, const float *__restrict__ w,
                                                 const ST *__restrict__ g, ST *__restrict__ v,
                                                 float *__restrict__ part, int H, int W)
{
    static_assert(TILE || std::is_same<ST, float>::value, "other storage types go through the LDS tile");
    extern __shared__ float smem[];
    constexpr int NCOL = C * K * K;            // shifted-x columns (i, a, b)
    constexpr int NS = (NCOL + 3) / 4;         // groups of four columns
    constexpr int P = C * NCOL;
    const int XR = H + K - 1, XW = W + K - 1;
    float *sv = smem;                          // [C][H][W]
    float *sx = sv + C * H * W;                // [C][XR][XW], origin at (-(K-1), -(K-1))
    float *sred = smem;                        // [4*64][NS*4], reuses the tiles after the products
    const int n = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;

    if constexpr (SPLIT) {
        // all waves stage x before the solve: eight loads in flight per thread, addresses clamped (no
        // branch around a load), halo zeroed when written; 16 bytes per load when the halo is four
        // columns and the rows are 16-byte aligned
        const float *xi = x + (size_t)n * C * H * W;
        if (K == 5 && (W & 3) == 0 && ((size_t)xi & 15) == 0 && ((C * H * W) & 3) == 0) {
            const int X4 = XW >> 2, total4 = C * XR * X4;
            for (int base = tid; base < total4; base += 8 * 256) {
                float4 val[8];
                bool halo[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int raw = base + u * 256;
                    const int idx = raw < total4 ? raw : total4 - 1;
                    const int c4 = idx % X4, rr = (idx / X4) % XR, ch = idx / (X4 * XR);
                    const int gr = rr - (K - 1), gc = 4 * c4 - (K - 1);
                    halo[u] = gr < 0 || gc < 0;
                    val[u] = *reinterpret_cast<const float4 *>(xi + (ch * H + (gr < 0 ? 0 : gr)) * W + (gc < 0 ? 0 : gc));
                }
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (base + u * 256 < total4)
                        *reinterpret_cast<float4 *>(sx + 4 * (base + u * 256)) =
                            halo[u] ? make_float4(0.f, 0.f, 0.f, 0.f) : val[u];
            }
        } else {
            const int total = C * XR * XW;
            for (int base = tid; base < total; base += 8 * 256) {
                float val[8];
                bool halo[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int raw = base + u * 256;
                    const int idx = raw < total ? raw : total - 1;
                    const int cc = idx % XW, rr = (idx / XW) % XR, ch = idx / (XW * XR);
                    const int gr = rr - (K - 1), gc = cc - (K - 1);
                    halo[u] = gr < 0 || gc < 0;
                    val[u] = xi[(ch * H + (gr < 0 ? 0 : gr)) * W + (gc < 0 ? 0 : gc)];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (base + u * 256 < total)
                        sx[base + u * 256] = halo[u] ? 0.0f : val[u];
            }
        }
        WaveSplitLds sl;
        sl.x = smem + ((C * H * W + C * XR * XW + 3) & ~3);     // 16-byte aligned behind the tiles
        sl.m = reinterpret_cast<f32x4 *>(sl.x + 2 * C * 64);
        solve_wave_split_body<C, K, 1, true>(g, w, v, H, W, n, sv, sl);
    } else if constexpr (TILE) {
        const ST *gi = g + (size_t)n * C * H * W;
        float4 *sv4 = reinterpret_cast<float4 *>(sv);
        const int n4 = C * H * W / 4;
        for (int i = tid; i < n4; i += 256)
            sv4[i] = ld4<ST>(gi, i);
        const ST *xi = x + (size_t)n * C * H * W;
        for (int idx = tid; idx < C * XR * XW; idx += 256) {
            const int cc = idx % XW, rr = (idx / XW) % XR, ch = idx / (XW * XR);
            const int gr = rr - (K - 1), gc = cc - (K - 1);
            sx[idx] = (gr >= 0 && gc >= 0) ? ld1(xi + (ch * H + gr) * W + gc) : 0.0f;
        }
        __syncthreads();
        if (wave == 0)
            solve_wave_body<C, K, 1, false, false, true>(nullptr, w, nullptr, H, W, n, sv);
    } else if (wave == 0) {
        solve_wave_body<C, K, 1, true>(g, w, v, H, W, n, sv);
    } else {
        const float *xi = x + (size_t)n * C * H * W;
        for (int idx = tid - 64; idx < C * XR * XW; idx += 192) {
            const int cc = idx % XW, rr = (idx / XW) % XR, ch = idx / (XW * XR);
            const int gr = rr - (K - 1), gc = cc - (K - 1);
            sx[idx] = (gr >= 0 && gc >= 0) ? xi[(ch * H + gr) * W + gc] : 0.0f;
        }
    }
    __syncthreads();
    if constexpr (TILE) {
        ST *vo = v + (size_t)n * C * H * W;
        const float4 *sv4 = reinterpret_cast<const float4 *>(sv);
        for (int i = tid; i < C * H * W / 4; i += 256)
            st4<ST>(vo, i, sv4[i]);
    }

    // lane = (block b, j): A row o = j, B column 4s + j.  Rows o >= C and columns
    // >= NCOL are padding: they read valid data (row/column 0) and their results
    // are never used.
    const int j = lane & 3, b = lane >> 2;
    const int aoff = (j < C) ? j * H * W : 0;
    int boff[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const int col = (4 * s + j < NCOL) ? 4 * s + j : 0;
        const int i = col / (K * K), a = (col / K) % K, bb = col % K;
        boff[s] = (i * XR + a) * XW + bb;
    }
    f32x4 acc[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s)
        acc[s] = f32x4{0.f, 0.f, 0.f, 0.f};
    if ((W & 15) == 0) {
        // rows are whole groups of 16 pixels: a wave takes rows wave, wave+4, ... and walks a row GPT
        // groups at a time, so that the tile offsets inside a trip are immediates
        auto rows_of = [&](auto gpt_tag) {
            constexpr int GPT = decltype(gpt_tag)::value;
            for (int pr = wave; pr < H; pr += 4) {
                const float *ap = sv + aoff + pr * W + b;
                const float *bp = sx + pr * XW + b;
                for (int pc = 0; pc < W; pc += 16 * GPT) {
                    float av[GPT];
#pragma unroll
                    for (int u = 0; u < GPT; ++u)
                        av[u] = ap[pc + 16 * u];
                    // group u+1's columns are read while group u's products run (NS independent accumulators)
                    float bv[2][NS];
#pragma unroll
                    for (int s = 0; s < NS; ++s)
                        bv[0][s] = bp[boff[s] + pc];
#pragma unroll
                    for (int u = 0; u < GPT; ++u) {
                        if (u + 1 < GPT) {
#pragma unroll
                            for (int s = 0; s < NS; ++s)
                                bv[(u + 1) & 1][s] = bp[boff[s] + pc + 16 * (u + 1)];
                        }
                        __builtin_amdgcn_sched_barrier(0);      // keep the reads ahead of the products below
#pragma unroll
                        for (int s = 0; s < NS; ++s)
                            acc[s] = __builtin_amdgcn_mfma_f32_4x4x1f32(av[u], bv[u & 1][s], acc[s], 0, 0, 0);
                    }
                }
            }
        };
        if ((W & 63) == 0)
            rows_of(std::integral_constant<int, 4>());
        else if ((W & 31) == 0)
            rows_of(std::integral_constant<int, 2>());
        else
            rows_of(std::integral_constant<int, 1>());
    } else {
        const int npix = H * W;
        const int ngroups = (npix + 15) / 16;
        for (int q = wave; q < ngroups; q += 4) {
            const int p = q * 16 + b;
            const bool pv = p < npix;
            const int pr = pv ? p / W : 0, pc = pv ? p - pr * W : 0;
            const float avl = sv[aoff + pr * W + pc];
            const float av = pv ? avl : 0.0f;       // pixels past the end contribute nothing
            const float *bp = sx + pr * XW + pc;
#pragma unroll
            for (int s = 0; s < NS; ++s)
                acc[s] = __builtin_amdgcn_mfma_f32_4x4x1f32(av, bp[boff[s]], acc[s], 0, 0, 0);
        }
    }
    __syncthreads();        // tiles no longer needed: reuse them for the reduction
    // lane (b, j) register (s, o) holds block b's partial of entry (o, col = 4s + j)
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int o = 0; o < 4; ++o)
            sred[tid * (NS * 4) + s * 4 + o] = acc[s][o];
    __syncthreads();
    // fixed-order sum in two levels: the 16 blocks of each wave, then the four waves
    float *swave = sred + 256 * NS * 4;     // [4][P]
    for (int idx = tid; idx < 4 * P; idx += 256) {
        const int e = idx % P, wv = idx / P;
        const int o = e / NCOL, col = e % NCOL;
        const int s = col >> 2, jj = col & 3;
        float sum = 0.0f;
#pragma unroll
        for (int bb = 0; bb < 16; ++bb)
            sum += sred[(wv * 64 + bb * 4 + jj) * (NS * 4) + s * 4 + o];
        swave[wv * P + e] = sum;
    }
    __syncthreads();
    for (int e = tid; e < P; e += 256)
        part[(size_t)n * P + e] = ((swave[e] + swave[P + e]) + swave[2 * P + e]) + swave[3 * P + e];
}

// Large batches of small images: the row-strided 4-byte accesses of all the resident waves keep
// B * rows * C * 2 cache lines of 128 bytes live; from about 16 MB on (the chip's L2s hold 32 MB, and
// not evenly) the image goes through LDS instead (k_solve_wave_tile), which moves whole lines:
// 3x32x32 forward, B = 4096: 140 -> 73 us; B = 1024: 38 -> 22 us; below that the plain kernels are
// faster (B = 256: 14.6 against 18.3 us, the copy in and out costs about 4 us of latency).
bool wave_tile_preferred(int B, int C, int H, int W)
{
    const size_t tile_bytes = (size_t)C * H * W * sizeof(float);
    const double live = (double)B * (H < 64 ? H : 64) * C * 256.0;
    return H <= 64 && live > 16.0 * 1024 * 1024 && tile_bytes <= 64 * 1024 && (C * H * W) % 4 == 0;
}

template <int C, int K>
static int launch_wave_ck(int dir, const float *in, const float *w, float *out, int B, int H, int W,
                          hipStream_t stream, float *logdet)
{
    // Large batches: every lane walks its own row 4 bytes at a time, so a wave keeps
    // rows * C * 2 (input and output) cache lines of 128 bytes live for dozens of steps.  When the
    // waves resident on the 32 CUs of an XCD need more than about 2.5 MB of its 4 MB L2, lines are
    // evicted between two touches and the solve becomes several times slower than running the batch
    // in rounds.  An LDS allocation the kernel never touches caps the waves per CU accordingly.
    size_t lds = 0;
    const size_t tile_bytes = (size_t)C * H * W * sizeof(float);
    // (two images per wave up to k = 7: beyond that the registers that hold the next pair would spill)
    if (K <= 7 && wave_tile_preferred(B, C, H, W) && H <= 32 && tile_bytes <= 16 * 64 * kTile2Pieces / 2 &&
        (((size_t)in | (size_t)out) & 15) == 0) {
        constexpr int KP = K <= 7 ? K : 3;      // (never launched for larger k; keeps those kernels out of the library)
        const size_t pair_bytes = 2 * tile_bytes + kTilePackPad * sizeof(float);
        const void *fn = dir ? reinterpret_cast<const void *>(&k_solve_wave_tile2<C, KP, 1>)
                             : reinterpret_cast<const void *>(&k_solve_wave_tile2<C, KP, 0>);
        // from four pairs per compute unit on: workgroups of four waves, as many as are resident at once
        const int npairs = (B + 1) / 2;
        int nw = 1, grid = npairs;
        if (4 * pair_bytes <= kMaxLdsBytes && ensure_dynamic_lds(fn, 4 * pair_bytes)) {
            const int resident = resident_workgroups(fn, 256, 4 * pair_bytes);
            if (resident > 0 && npairs >= 4 * resident) {
                nw = 4;
                grid = resident;
            }
        }
        if (!ensure_dynamic_lds(fn, nw * pair_bytes))
            return INVCONV_ERR_UNSUPPORTED;
        if (dir)
            hipLaunchKernelGGL((k_solve_wave_tile2<C, KP, 1>), dim3(grid), dim3(64 * nw), nw * pair_bytes, stream, in, w,
                               out, B, H, W, logdet);
        else
            hipLaunchKernelGGL((k_solve_wave_tile2<C, KP, 0>), dim3(grid), dim3(64 * nw), nw * pair_bytes, stream, in, w,
                               out, B, H, W, logdet);
        return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
    }
    if (wave_tile_preferred(B, C, H, W) && (((size_t)in | (size_t)out) & 15) == 0) {
        const void *fn = dir ? reinterpret_cast<const void *>(&k_solve_wave_tile<C, K, 1>)
                             : reinterpret_cast<const void *>(&k_solve_wave_tile<C, K, 0>);
        if (!ensure_dynamic_lds(fn, tile_bytes))
            return INVCONV_ERR_UNSUPPORTED;
        if (dir)
            hipLaunchKernelGGL((k_solve_wave_tile<C, K, 1>), dim3(B), dim3(64), tile_bytes, stream, in, w, out, H, W,
                               logdet);
        else
            hipLaunchKernelGGL((k_solve_wave_tile<C, K, 0>), dim3(B), dim3(64), tile_bytes, stream, in, w, out, H, W,
                               logdet);
        return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
    }
    if (B > 512) {
        const size_t live = (size_t)(H < 64 ? H : 64) * C * 2 * 128;
        size_t cap = (size_t)(2.5 * 1024 * 1024) / (32 * live);
        cap = cap < 1 ? 1 : cap;
        if (cap < 8) {
            lds = (kMaxLdsBytes / cap) & ~(size_t)255;
            const void *fn = dir ? reinterpret_cast<const void *>(&k_solve_wave<C, K, 1>)
                                 : reinterpret_cast<const void *>(&k_solve_wave<C, K, 0>);
            if (!ensure_dynamic_lds(fn, lds))
                lds = 0;
        }
    }
    if (dir)
        hipLaunchKernelGGL((k_solve_wave<C, K, 1>), dim3(B), dim3(64), lds, stream, in, w, out, H, W, logdet);
    else
        hipLaunchKernelGGL((k_solve_wave<C, K, 0>), dim3(B), dim3(64), lds, stream, in, w, out, H, W, logdet);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

static int wave_bands_log_steps(int W) { return (64 + W - 1 + kWavePF - 1) / kWavePF * kWavePF; }

static size_t wave_bands_lds_bytes(int H, int W, int k)
{
    const size_t nb = (H + 63) / 64;
    return ((nb - 1) * (size_t)wave_bands_log_steps(W) + 64) * (k - 1) * sizeof(f32x4) + nb * sizeof(int);
}

constexpr int kBandSpinLimit = 1 << 22;       // polls of an LDS counter (64 clocks apart)
constexpr int kCourierSpinLimit = 1 << 22;    // idle rounds of a courier wave

template <int C, int K>
static int launch_wave_bands_ck(int dir, const float *in, const float *w, float *out, int B, int H, int W,
                                hipStream_t stream, int *err)
{
    const int nb = (H + 63) / 64, log_steps = wave_bands_log_steps(W);
    const size_t lds = wave_bands_lds_bytes(H, W, K);
    if (lds > 128 * 1024)       // reached only when the multi-workgroup launch has no workspace to put its logs in
        return launch_solve_block(dir, in, w, out, B, C, H, W, K, stream);
    const void *fn = dir ? reinterpret_cast<const void *>(&k_solve_wave_bands<C, K, 1>)
                         : reinterpret_cast<const void *>(&k_solve_wave_bands<C, K, 0>);
    if (!ensure_dynamic_lds(fn, lds))
        return INVCONV_ERR_UNSUPPORTED;
    const int spin = wait_budget(kBandSpinLimit);
    if (dir)
        hipLaunchKernelGGL((k_solve_wave_bands<C, K, 1>), dim3(B), dim3(64 * nb), lds, stream, in, w, out, H, W,
                           log_steps, spin, err);
    else
        hipLaunchKernelGGL((k_solve_wave_bands<C, K, 0>), dim3(B), dim3(64 * nb), lds, stream, in, w, out, H, W,
                           log_steps, spin, err);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

// Bands on different compute units (k_solve_wave_bands_multi).  The logs and counters between workgroups
// live in the caller's workspace.  A band's workgroup waits for the one of the band above, so the images
// go out in launches of at most as many workgroups as the device holds at once: inside a launch nothing
// depends on the order in which the hardware starts workgroups.
static size_t wave_bands_multi_ws_per_image(int H, int W, int k)
{
    const size_t nb = (H + 63) / 64;
    return (nb - 1) * ((size_t)wave_bands_log_steps(W) * (k - 1) * sizeof(f32x4) + 256);
}

static bool wave_bands_single_fits(int H, int W, int k) { return wave_bands_lds_bytes(H, W, k) <= 128 * 1024; }
static bool wave_bands_multi_strided_pays(int B, int H, int W)
{
    const int nb = (H + 63) / 64;
    return nb >= 3 && W >= 128 && (long)B * nb <= 512;
}

static size_t wave_bands_io_lds_bytes(int C, int W, int k)
{
    return (2 * (size_t)wave_bands_log_steps(W) + 64) * (k - 1) * sizeof(f32x4) +
           (size_t)C * 64 * kRingStride * sizeof(float) + 6 * sizeof(int);
}

template <int C, int K>
static int launch_wave_bands_multi_ck(int dir, const float *in, const float *w, float *out, int B, int H, int W,
                                      hipStream_t stream, SolveWs ws)
{
    const int nb = (H + 63) / 64, log_steps = wave_bands_log_steps(W);
    const size_t seg = (size_t)log_steps * (K - 1);
    // rows through an LDS ring (whole-line memory traffic) where rows are made of 16-byte pieces
    const size_t lds_io = wave_bands_io_lds_bytes(C, W, K);
    const bool io = (W & 3) == 0 && lds_io <= kMaxLdsBytes &&
                    ((reinterpret_cast<uintptr_t>(in) | reinterpret_cast<uintptr_t>(out)) & 15) == 0;
    if (!io && wave_bands_single_fits(H, W, K) && !wave_bands_multi_strided_pays(B, H, W))
        return launch_wave_bands_ck<C, K>(dir, in, w, out, B, H, W, stream, ws.err);
    const size_t lds = io ? lds_io : (2 * seg + 64 * (K - 1)) * sizeof(f32x4) + 2 * sizeof(int);
    const void *fn = io ? (dir ? reinterpret_cast<const void *>(&k_solve_wave_bands_io<C, K, 1>)
                               : reinterpret_cast<const void *>(&k_solve_wave_bands_io<C, K, 0>))
                        : (dir ? reinterpret_cast<const void *>(&k_solve_wave_bands_multi<C, K, 1>)
                               : reinterpret_cast<const void *>(&k_solve_wave_bands_multi<C, K, 0>));
    if (!ensure_dynamic_lds(fn, lds))
        return INVCONV_ERR_UNSUPPORTED;
    const int resident = resident_workgroups(fn, io ? 256 : 128, lds);
    int per_launch = resident / nb;                 // images per launch
    if (per_launch < 1)
        return launch_wave_bands_ck<C, K>(dir, in, w, out, B, H, W, stream, ws.err);
    if (per_launch > B)
        per_launch = B;
    // workspace: counters of all images of a launch, then their logs; launches follow each other on the
    // stream, so they share the space, and a small workspace only means more launches
    const size_t per_image = wave_bands_multi_ws_per_image(H, W, K);
    const size_t fit = ws.base ? ws.bytes / per_image : 0;
    if ((size_t)per_launch > fit)
        per_launch = (int)fit;
    if (per_launch < 1)
        return launch_wave_bands_ck<C, K>(dir, in, w, out, B, H, W, stream, ws.err);
    const size_t ncnt = (size_t)per_launch * (nb - 1);
    const size_t cnt_bytes = (ncnt * sizeof(int) + 255) / 256 * 256;     // at most 256 bytes per counter: fits
    int *gcount = reinterpret_cast<int *>(ws.base);
    f32x4 *glog = reinterpret_cast<f32x4 *>(ws.base + cnt_bytes);
    const int spin_courier = wait_budget(kCourierSpinLimit);
    const size_t img = (size_t)C * H * W;
    for (int n0 = 0; n0 < B; n0 += per_launch) {
        const int nimg = B - n0 < per_launch ? B - n0 : per_launch;
        const int cnt = nimg * (nb - 1);
        hipLaunchKernelGGL(k_wave_bands_clear, dim3((unsigned)((cnt + 255) / 256)), dim3(256), 0, stream, gcount, cnt);
        const dim3 grid((unsigned)(nimg * nb));    // band-major: a band's workgroups come after those it waits for
        if (io) {
            const int spin_band = wait_budget(kBandSpinLimit);
            if (dir)
                hipLaunchKernelGGL((k_solve_wave_bands_io<C, K, 1>), grid, dim3(256), lds, stream, in + n0 * img, w,
                                   out + n0 * img, nimg, H, W, log_steps, gcount, glog, spin_band, spin_courier,
                                   ws.err);
            else
                hipLaunchKernelGGL((k_solve_wave_bands_io<C, K, 0>), grid, dim3(256), lds, stream, in + n0 * img, w,
                                   out + n0 * img, nimg, H, W, log_steps, gcount, glog, spin_band, spin_courier,
                                   ws.err);
        } else if (dir)
            hipLaunchKernelGGL((k_solve_wave_bands_multi<C, K, 1>), grid, dim3(128), lds, stream, in + n0 * img, w,
                               out + n0 * img, nimg, H, W, log_steps, gcount, glog, spin_courier, ws.err);
        else
            hipLaunchKernelGGL((k_solve_wave_bands_multi<C, K, 0>), grid, dim3(128), lds, stream, in + n0 * img, w,
                               out + n0 * img, nimg, H, W, log_steps, gcount, glog, spin_courier, ws.err);
        if (hipGetLastError() != hipSuccess)
            return INVCONV_ERR_LAUNCH;
    }
    return INVCONV_OK;
}

// Several compute units per image.  With the solving wave reading its rows itself (k_solve_wave_bands_multi)
// this pays while there are compute units to spare and an image has at least three bands of some width: the
// bands of an image are then limited by the address unit of the one compute unit they share (0.49 us per
// step at 3x256x256 against 0.31 us), while the hand-over through global memory makes a band trail the one
// above by about 105 steps instead of 80.  With the rows passing through the LDS ring (k_solve_wave_bands_io,
// rows of 16-byte pieces) it pays at every batch size from 64 columns on, since the memory instructions no
// longer touch 64 lines each (measured forward + backward, ring against one workgroup per image:
// 128 x 3x256x256 448 us against 868, 256 x 3x128x128 228 against 354, 1024 x 3x96x96 695 against 1725,
// 256 x 3x128x64 179 against 190; 256 x 3x192x32 392 against 217, hence the lower limit on the width).
// Images whose logs do not fit one workgroup's LDS (3x512x512) have only these two ways.
static size_t wave_bands_multi_lds_bytes(int W, int k)
{
    return (2 * (size_t)wave_bands_log_steps(W) + 64) * (k - 1) * sizeof(f32x4) + 2 * sizeof(int);
}
static bool wave_bands_multi_preferred(int B, int H, int W, int k)
{
    if (wave_bands_multi_lds_bytes(W, k) > kMaxLdsBytes)
        return false;
    if (!wave_bands_single_fits(H, W, k))
        return true;
    if ((W & 3) == 0 && W >= 64 && wave_bands_io_lds_bytes(4, W, k) <= kMaxLdsBytes)
        return true;        // rows through the LDS ring (k_solve_wave_bands_io)
    return wave_bands_multi_strided_pays(B, H, W);
}

// The four-wave split of the solve costs about a microsecond more before its first step and saves
// 20 ns (k = 3) to 140 ns (k = 5) per step at up to 32 rows, less at 64.  The forward launch uses it
// unless the image is tiny or the batch large enough to fill the CUs with single waves.  Inside the
// fused backward kernel it pays for k = 5 only: there the single wave leaves the other three free to
// stage x meanwhile, which the split has to do before it starts (measured at k = 3: 2.6 us slower).
static bool wave_split_pays(int k) { return k >= 5; }

bool wave_split_preferred(int B, int H, int W, int k) { return k >= 3 && (k >= 5 || H + W >= 48) && B <= 512; }

// ---------------------------------------------------------------------------
// The backward pass of one image on eight waves (W a multiple of 16, at most 64): waves 0..3 run the
// transposed solve with its steps split over them (solve_wave_split_body, which also keeps dL/dy in an
// LDS tile), waves 4..7 meanwhile stage x and then form the weight-gradient products behind the
// wavefront: mirrored row r of dL/dy is complete in LDS once step r + W has ended, a row goes to helper
// wave r mod 4, and a helper takes one group of 16 pixels per step, so it keeps up with the solve.  The
// helpers pass through the same barriers as the solving waves (one after the set-up, one per step),
// doing a slice of their work in between.  What is left after the last step (the rows of
// the last few steps) is finished by the helpers before the common reduction.
// ---------------------------------------------------------------------------
template <int C, int K>
__global__ __launch_bounds__(512) void k_bwd_wave8(const float *__restrict__ x, const float *__restrict__ w,
                                                  const float *__restrict__ g, float *__restrict__ v,
                                                  float *__restrict__ part, int H, int W)
{
    extern __shared__ float smem[];
    constexpr int NCOL = C * K * K;            // shifted-x columns (i, a, b)
    constexpr int NS = (NCOL + 3) / 4;         // groups of four columns
    constexpr int P = C * NCOL;
    const int XR = H + K - 1, XW = W + K - 1;
    float *sv = smem;                          // [C][H][W]
    float *sx = sv + C * H * W;                // [C][XR][XW], origin at (-(K-1), -(K-1))
    float *sred = smem;                        // [4*64][NS*4], reuses the tiles after the products
    const int n = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    if (wave < 4) {
        __builtin_amdgcn_s_setprio(2);      // the dependent chain goes first; the helpers fill the gaps
        WaveSplitLds sl;
        sl.x = smem + ((C * H * W + C * XR * XW + 3) & ~3);     // 16-byte aligned behind the tiles
        sl.m = reinterpret_cast<f32x4 *>(sl.x + 2 * C * 64);
        solve_wave_split_body<C, K, 1, true>(g, w, v, H, W, n, sv, sl);
        __syncthreads();        // the helpers have finished the products
    } else {
        const int ht = tid - 256, hw = wave - 4;
        const float *xi = x + (size_t)n * C * H * W;
        for (int base = ht; base < C * XR * XW; base += 8 * 256) {
            float val[8];
            bool halo[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int raw = base + u * 256;
                const int idx = raw < C * XR * XW ? raw : C * XR * XW - 1;
                const int cc = idx % XW, rr = (idx / XW) % XR, ch = idx / (XW * XR);
                const int gr = rr - (K - 1), gc = cc - (K - 1);
                halo[u] = gr < 0 || gc < 0;
                val[u] = xi[(ch * H + (gr < 0 ? 0 : gr)) * W + (gc < 0 ? 0 : gc)];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (base + u * 256 < C * XR * XW)
                    sx[base + u * 256] = halo[u] ? 0.0f : val[u];
        }
        // lane = (block b, j): A row o = j, B column 4s + j (padding rows / columns read valid data, unused)
        const int j = lane & 3, b = lane >> 2;
        const int aoff = (j < C) ? j * H * W : 0;
        int boff[NS];
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const int col = (4 * s + j < NCOL) ? 4 * s + j : 0;
            const int i = col / (K * K), a = (col / K) % K, bb = col % K;
            boff[s] = (i * XR + a) * XW + bb;
        }
        f32x4 acc[NS];
#pragma unroll
        for (int s = 0; s < NS; ++s)
            acc[s] = f32x4{0.f, 0.f, 0.f, 0.f};
        // one group: 16 pixels pc .. pc+15 of image row pr
        auto group = [&](int pr, int pc) {
            const float av = sv[aoff + pr * W + b + pc];
            const float *bp = sx + pr * XW + b + pc;
            float bv[NS];
#pragma unroll
            for (int s = 0; s < NS; ++s)
                bv[s] = bp[boff[s]];
#pragma unroll
            for (int s = 0; s < NS; ++s)
                acc[s] = __builtin_amdgcn_mfma_f32_4x4x1f32(av, bv[s], acc[s], 0, 0, 0);
        };
        const int ngrp = W >> 4;
        int row = hw, grp = 0;                  // next group of this helper: mirrored row `row`, group `grp`
        __syncthreads();        // the solving waves' set-up barrier; x is staged for all helpers
        const int total = H + W - 1 + 2;
        for (int s = -1; s < total - 1; ++s) {
            // mirrored row r is complete once step r + W has ended, i.e. from step r + W + 1 on
            if (row < H && row + W + 1 <= s) {
                group(H - 1 - row, 16 * grp);
                if (++grp == ngrp) {
                    grp = 0;
                    row += 4;
                }
            }
            __syncthreads();
        }
        // (the last step's barrier has passed: every row is complete)
        while (row < H) {
            group(H - 1 - row, 16 * grp);
            if (++grp == ngrp) {
                grp = 0;
                row += 4;
            }
        }
        __syncthreads();        // products finished: the tiles can be reused
        // lane (b, j) register (s, o) holds block b's partial of entry (o, col = 4s + j)
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int o = 0; o < 4; ++o)
                sred[ht * (NS * 4) + s * 4 + o] = acc[s][o];
    }
    __syncthreads();
    // fixed-order sum in two levels: the 16 blocks of each helper wave, then the four helper waves
    float *swave = sred + 256 * NS * 4;     // [4][P]
    for (int idx = tid; idx < 4 * P; idx += 512) {
        const int e = idx % P, wv = idx / P;
        const int o = e / NCOL, col = e % NCOL;
        const int s = col >> 2, jj = col & 3;
        float sum = 0.0f;
#pragma unroll
        for (int bb = 0; bb < 16; ++bb)
            sum += sred[(wv * 64 + bb * 4 + jj) * (NS * 4) + s * 4 + o];
        swave[wv * P + e] = sum;
    }
    __syncthreads();
    for (int e = tid; e < P; e += 512)
        part[(size_t)n * P + e] = ((swave[e] + swave[P + e]) + swave[2 * P + e]) + swave[3 * P + e];
}

// ---------------------------------------------------------------------------
// Backward pass of a whole flow step for few channels and few images, on the same eight waves: the inputs are z
// and dL/dz.  Waves 0..3 run the transposed solve on dL/dz with A^T folded into its input weights; waves 4..7
// stage x = A^-1 z - b/s (zero halo) and dL/dz in LDS and form, behind the wavefront, the outer products of the
// weight gradient and, with dL/dz as the first operand, M2[o][i] = sum dL/dz[o] x[i] and m1[o] = sum dL/dz[o].
// One row [P | C*C | C] per image, fixed-order sums; no set-up launch (the waves form the small matrices
// themselves).
// ---------------------------------------------------------------------------
template <int C, int K>
__global__ __launch_bounds__(512) void k_flow_bwd_wave8(const float *__restrict__ z, const float *__restrict__ w,
                                                       const float *__restrict__ gz, FlowParams fp,
                                                       float *__restrict__ v, float *__restrict__ part, int H, int W)
{
    extern __shared__ float smem[];
    constexpr int NCOL = C * K * K, NS = (NCOL + 3) / 4, P = C * NCOL;
    constexpr int NC2 = C + 1, NS2 = (NC2 + 3) / 4, P2 = C * NC2;       // second operand: x[i] of the pixel, and 1
    constexpr int NST = NS + NS2, PT = P + P2;
    const int XR = H + K - 1, XW = W + K - 1, HW = H * W;
    float *sv = smem;                          // [C][H][W]   dL/dy as the solve completes it
    float *sx = sv + C * HW;                   // [C][XR][XW] x, origin at (-(K-1), -(K-1))
    float *sg = sx + C * XR * XW;              // [C][H][W]   dL/dz
    float *sred = smem;                        // [4*64][NST*4], reuses the tiles after the products
    const int n = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    if (wave < 4) {
        __builtin_amdgcn_s_setprio(2);      // the dependent chain goes first; the helpers fill the gaps
        WaveSplitLds sl;
        sl.x = smem + ((2 * C * HW + C * XR * XW + 3) & ~3);    // 16-byte aligned behind the tiles
        sl.m = reinterpret_cast<f32x4 *>(sl.x + 2 * C * 64);
        solve_wave_split_body<C, K, 1, true, 2, true>(gz, w, v, H, W, n, sv, sl, fp);
        __syncthreads();        // the helpers have finished the products
    } else {
        const int ht = tid - 256, hw = wave - 4;
        // A^-1 = diag(1/s) Q^-1 and e = -b/s
        float Ai[C][C], ev[C];
        {
            double q[C][C], qi[C][C];
#pragma unroll
            for (int o = 0; o < C; ++o)
#pragma unroll
                for (int i = 0; i < C; ++i)
                    q[o][i] = (double)fp.Q[o * C + i];
            small_det_inv<C>(q, qi);
#pragma unroll
            for (int i = 0; i < C; ++i) {
                ev[i] = -fp.b[i] / fp.s[i];
#pragma unroll
                for (int o = 0; o < C; ++o)
                    Ai[i][o] = (float)(qi[i][o] / (double)fp.s[i]);
            }
        }
        const float *zi = z + (size_t)n * C * HW, *gi = gz + (size_t)n * C * HW;
        // a thread takes positions of the padded x tile, four at a time: all channels of z and dL/dz of the pixel
        for (int base = ht; base < XR * XW; base += 4 * 256) {
            float zv[4][C], gv[4][C];
            bool halo[4];
            int gpix[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int raw = base + u * 256;
                const int idx = raw < XR * XW ? raw : XR * XW - 1;
                const int cc = idx % XW, rr = idx / XW;
                const int gr = rr - (K - 1), gc = cc - (K - 1);
                halo[u] = gr < 0 || gc < 0;
                gpix[u] = (gr < 0 ? 0 : gr) * W + (gc < 0 ? 0 : gc);
#pragma unroll
                for (int c = 0; c < C; ++c) {
                    zv[u][c] = zi[c * HW + gpix[u]];
                    gv[u][c] = gi[c * HW + gpix[u]];
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int raw = base + u * 256;
                if (raw < XR * XW) {
#pragma unroll
                    for (int i = 0; i < C; ++i) {
                        float xi = ev[i];
#pragma unroll
                        for (int o = 0; o < C; ++o)
                            xi += Ai[i][o] * zv[u][o];
                        sx[i * XR * XW + raw] = halo[u] ? 0.0f : xi;
                        if (!halo[u])
                            sg[i * HW + gpix[u]] = gv[u][i];
                    }
                }
            }
        }
        // lane = (block b, j): first operand row o = j (of dL/dy, or of dL/dz), second operand column 4s + j
        // (padding rows / columns read valid data, unused)
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
        // one group: 16 pixels pc .. pc+15 of image row pr
        auto group = [&](int pr, int pc) {
            const float av = sv[aoff + pr * W + b + pc], ag = sg[aoff + pr * W + b + pc];
            const float *bp = sx + pr * XW + b + pc;
            float bv[NST];
#pragma unroll
            for (int s = 0; s < NST; ++s)
                bv[s] = bp[boff[s]];
#pragma unroll
            for (int s = 0; s < NS; ++s)
                acc[s] = __builtin_amdgcn_mfma_f32_4x4x1f32(av, bv[s], acc[s], 0, 0, 0);
#pragma unroll
            for (int s = 0; s < NS2; ++s)
                acc[NS + s] = __builtin_amdgcn_mfma_f32_4x4x1f32(ag, one[s] ? 1.0f : bv[NS + s], acc[NS + s], 0, 0, 0);
        };
        const int ngrp = W >> 4;
        int row = hw, grp = 0;                  // next group of this helper: mirrored row `row`, group `grp`
        __syncthreads();        // the solving waves' set-up barrier; x and dL/dz are staged for all helpers
        const int total = H + W - 1 + 2;
        for (int s = -1; s < total - 1; ++s) {
            // mirrored row r is complete once step r + W has ended, i.e. from step r + W + 1 on
            if (row < H && row + W + 1 <= s) {
                group(H - 1 - row, 16 * grp);
                if (++grp == ngrp) {
                    grp = 0;
                    row += 4;
                }
            }
            __syncthreads();
        }
        // (the last step's barrier has passed: every row is complete)
        while (row < H) {
            group(H - 1 - row, 16 * grp);
            if (++grp == ngrp) {
                grp = 0;
                row += 4;
            }
        }
        __syncthreads();        // products finished: the tiles can be reused
#pragma unroll
        for (int s = 0; s < NST; ++s)
#pragma unroll
            for (int o = 0; o < 4; ++o)
                sred[ht * (NST * 4) + s * 4 + o] = acc[s][o];
    }
    __syncthreads();
    // fixed-order sum in two levels: the 16 blocks of each helper wave, then the four helper waves
    float *swave = sred + 256 * NST * 4;     // [4][PT]
    for (int idx = tid; idx < 4 * PT; idx += 512) {
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
    for (int e = tid; e < PT; e += 512) {
        const float val = ((swave[e] + swave[PT + e]) + swave[2 * PT + e]) + swave[3 * PT + e];
        int dst = e;
        if (e >= P) {
            const int o = (e - P) / NC2, col = (e - P) % NC2;
            dst = col < C ? P + o * C + col : P + C * C + o;
        }
        part[(size_t)n * PT + dst] = val;
    }
}

static size_t flow_bwd_wave8_lds_bytes(int C, int H, int W, int k)
{
    const size_t tiles = 2 * (size_t)C * H * W + (size_t)C * (H + k - 1) * (W + k - 1) + 4 + 2 * (size_t)C * 64 +
                         2 * (size_t)k * 64 * 4;
    const size_t nst = (size_t)(C * k * k + 3) / 4 + (size_t)(C + 1 + 3) / 4;
    const size_t red = 256 * nst * 4 + 4 * ((size_t)C * C * k * k + (size_t)C * (C + 1));
    return sizeof(float) * (tiles > red ? tiles : red);
}

// few channels, k = 3, few images of rows made of whole 16-pixel groups: the shapes of k_bwd_wave8
bool flow_bwd_split_supported(int B, int C, int H, int W, int k)
{
    return C >= 1 && C <= 4 && k == 3 && wave_supported(C, H, k) && B <= 256 && (W & 15) == 0 && W <= 64 &&
           !wave_tile_preferred(B, C, H, W) && flow_bwd_wave8_lds_bytes(C, H, W, k) <= kMaxLdsBytes;
}

template <int C>
static int launch_flow_bwd_split_c(const float *z, const float *w, const float *gz, FlowParams fp, float *v,
                                   float *part, int B, int H, int W, hipStream_t stream)
{
    const size_t lds = flow_bwd_wave8_lds_bytes(C, H, W, 3);
    if (!ensure_dynamic_lds(reinterpret_cast<const void *>(&k_flow_bwd_wave8<C, 3>), lds))
        return INVCONV_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((k_flow_bwd_wave8<C, 3>), dim3(B), dim3(512), lds, stream, z, w, gz, fp, v, part, H, W);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

// dL/dy and one row [C*C*k*k | C*C | C] per image (un-negated dL/dw sums, M2, m1) in one launch
int launch_flow_bwd_split(const float *z, const float *w, const float *gz, const float *s, const float *b,
                          const float *Q, float *v, float *part, int B, int C, int H, int W, int k, hipStream_t stream)
{
    if (!flow_bwd_split_supported(B, C, H, W, k))
        return INVCONV_ERR_VARIANT;
    const FlowParams fp{s, b, Q};
    switch (C) {
    case 1: return launch_flow_bwd_split_c<1>(z, w, gz, fp, v, part, B, H, W, stream);
    case 2: return launch_flow_bwd_split_c<2>(z, w, gz, fp, v, part, B, H, W, stream);
    case 3: return launch_flow_bwd_split_c<3>(z, w, gz, fp, v, part, B, H, W, stream);
    default: return launch_flow_bwd_split_c<4>(z, w, gz, fp, v, part, B, H, W, stream);
    }
}

size_t bwd_wave_lds_bytes(int C, int H, int W, int k)
{
    size_t tiles = (size_t)C * H * W + (size_t)C * (H + k - 1) * (W + k - 1);
    if (wave_split_pays(k))
        tiles += 4 + 2 * (size_t)C * 64 + 2 * (size_t)k * 64 * 4;      // exchange buffers of the split solve
    const size_t red = 256 * (size_t)((C * k * k + 3) / 4) * 4 + 4 * (size_t)C * C * k * k;
    return sizeof(float) * (tiles > red ? tiles : red);
}

static size_t bwd_wave8_lds_bytes(int C, int H, int W, int k)
{
    const size_t tiles = (size_t)C * H * W + (size_t)C * (H + k - 1) * (W + k - 1) + 4 + 2 * (size_t)C * 64 +
                         2 * (size_t)k * 64 * 4;
    const size_t red = 256 * (size_t)((C * k * k + 3) / 4) * 4 + 4 * (size_t)C * C * k * k;
    return sizeof(float) * (tiles > red ? tiles : red);
}

template <int C, int K>
static int launch_bwd_wave_ck(const float *x, const float *w, const float *g, float *v, float *part, int B, int H,
                              int W, hipStream_t stream)
{
    const size_t lds = bwd_wave_lds_bytes(C, H, W, K);
    constexpr bool kSplit = K >= 5;
    if (!ensure_dynamic_lds(reinterpret_cast<const void *>(&k_bwd_wave<C, K, kSplit>), lds))
        return INVCONV_ERR_UNSUPPORTED;
    if (!kSplit && wave_tile_preferred(B, C, H, W) && (((size_t)g | (size_t)v) & 15) == 0) {
        if (!ensure_dynamic_lds(reinterpret_cast<const void *>(&k_bwd_wave<C, K, false, true>), lds))
            return INVCONV_ERR_UNSUPPORTED;
        hipLaunchKernelGGL((k_bwd_wave<C, K, false, true>), dim3(B), dim3(256), lds, stream, x, w, g, v, part, H, W);
        return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
    }
    if constexpr (K == 3) {
        // eight waves while every image still gets a compute unit's worth of waves (k = 3: headline backward
        // 20.4 -> 19.7 us; at k = 5 the same arrangement measured 3.5 us slower than four waves): the products run behind the solve instead of after it (rows of whole 16-pixel groups,
        // at most four per row, so that a helper wave keeps up with one group per step)
        const size_t lds8 = bwd_wave8_lds_bytes(C, H, W, K);
        if (B <= 256 && (W & 15) == 0 && W <= 64 && lds8 <= kMaxLdsBytes) {
            if (!ensure_dynamic_lds(reinterpret_cast<const void *>(&k_bwd_wave8<C, K>), lds8))
                return INVCONV_ERR_UNSUPPORTED;
            hipLaunchKernelGGL((k_bwd_wave8<C, K>), dim3(B), dim3(512), lds8, stream, x, w, g, v, part, H, W);
            return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
        }
    }
    hipLaunchKernelGGL((k_bwd_wave<C, K, kSplit>), dim3(B), dim3(256), lds, stream, x, w, g, v, part, H, W);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

// The fused kernel gives a whole workgroup to every image while only one of its waves solves, and registers
// and LDS allow at most three such workgroups per compute unit.  Once a large batch needs more than about
// 1.3 rounds of them, the transposed solve as a launch of its own (one wave per image, or per two) followed
// by the streaming weight-gradient kernel is faster: 3x32x32, B = 1400: 53 against 67 us, B = 4096: 91
// against 159 us; 3x64x64, B = 400: 65 against 122 us; 1x28x28, B = 4096: 49 against 63 us; B = 1024 at
// 3x32x32 is a tie, 700 still favours the fused kernel (38 against 43 us).
bool bwd_wave_fused_pays(int B, int C, int H, int W, int k)
{
    if (!wave_tile_preferred(B, C, H, W))
        return true;
    const size_t lds = bwd_wave_lds_bytes(C, H, W, k);
    size_t per_cu = lds ? kMaxLdsBytes / lds : 3;
    per_cu = per_cu > 3 ? 3 : (per_cu < 1 ? 1 : per_cu);
    return (double)B <= 1.3 * (double)per_cu * 256.0;      // 256 compute units
}

bool bwd_wave_supported(int C, int H, int W, int k)
{
    // (k = 5 and 7 used to run here with the split solve inside; the split solve as a launch of its own followed by
    // the weight-gradient kernels is as fast or faster: 32 x 3x64x64 k = 5 55 -> 45 us, 16 x 3x32x32 k = 7 50 -> 38 us)
    return wave_supported(C, H, k) && k <= 3 && bwd_wave_lds_bytes(C, H, W, k) <= kMaxLdsBytes;
}

// dL/dy and the per-image partial sums of dL/dw (part[B][C*C*k*k], un-negated) in one launch.
int launch_bwd_wave(const float *x, const float *w, const float *g, float *v, float *part, int B, int C, int H,
                    int W, int k, hipStream_t stream)
{
    if (!bwd_wave_supported(C, H, W, k))
        return INVCONV_ERR_VARIANT;
    if (C == 3 && k == 3) return launch_bwd_wave_ck<3, 3>(x, w, g, v, part, B, H, W, stream);
    if (C == 3 && k == 2) return launch_bwd_wave_ck<3, 2>(x, w, g, v, part, B, H, W, stream);
    if (C == 1 && k == 3) return launch_bwd_wave_ck<1, 3>(x, w, g, v, part, B, H, W, stream);
    if (C == 2 && k == 3) return launch_bwd_wave_ck<2, 3>(x, w, g, v, part, B, H, W, stream);
    if (C == 4 && k == 3) return launch_bwd_wave_ck<4, 3>(x, w, g, v, part, B, H, W, stream);
    return INVCONV_ERR_VARIANT;
}

// Kernel sizes of the paper's kernel-size ablation (2, 3, 5, 7, 9, 11) for three channels.  Registers hold
// every folded tap, so the larger kernels exist for the solve only: the fused backward kernel stops at
// k = 7 and the banded one at k = 5 (beyond that they would spill to scratch memory).
static bool wave_ck(int C, int k)
{
    return (C == 3 && (k == 2 || k == 3 || k == 5 || k == 7 || k == 9 || k == 11)) || (C == 1 && k == 3) ||
           (C == 2 && k == 3) || (C == 4 && k == 3);
}

bool wave_supported(int C, int H, int k) { return H <= 64 && wave_ck(C, k); }

// 65 .. 512 rows, bands of 64 rows; the message log of the band boundaries has to fit LDS
bool wave_bands_supported(int C, int H, int W, int k)
{
    return H > 64 && H <= 512 && wave_ck(C, k) && k <= 5 &&
           (wave_bands_lds_bytes(H, W, k) <= 128 * 1024 ||
            (2 * (size_t)wave_bands_log_steps(W) + 64) * (k - 1) * sizeof(f32x4) + 2 * sizeof(int) <= kMaxLdsBytes);
}

template <int C, int K>
static int launch_wave_split_ck(int dir, const float *in, const float *w, float *out, int B, int H, int W,
                                hipStream_t stream, float *logdet)
{
    const dim3 block(64 * (wave_split_nf(K) + 2));
    if (dir)
        hipLaunchKernelGGL((k_solve_wave_split<C, K, 1>), dim3(B), block, 0, stream, in, w, out, H, W, logdet);
    else
        hipLaunchKernelGGL((k_solve_wave_split<C, K, 0>), dim3(B), block, 0, stream, in, w, out, H, W, logdet);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

// Same shapes as the single-wave kernel; four to seven waves per image.
// The flow step's forward pass on the split solve: the shapes of the fused flow kernels (few channels, k = 3, or
// three channels and k = 5) while the split solve is the better single-layer kernel (few images).
bool flow_split_supported(int B, int C, int H, int W, int k)
{
    const bool ck = (C == 3 && (k == 3 || k == 5)) || ((C == 1 || C == 2 || C == 4) && k == 3);
    return ck && wave_supported(C, H, k) && wave_split_preferred(B, H, W, k) && !wave_tile_preferred(B, C, H, W);
}

template <int C, int K>
static int launch_flow_fwd_split_ck(const float *y, const float *w, FlowParams fp, float *z, int B, int H, int W,
                                    hipStream_t stream, float *logdet)
{
    hipLaunchKernelGGL((k_flow_fwd_split<C, K>), dim3(B), dim3(64 * (wave_split_nf(K) + 2)), 0, stream, y, w, fp, z, H,
                       W, logdet);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

int launch_flow_fwd_split(const float *y, const float *w, const float *s, const float *b, const float *Q, float *z,
                          int B, int C, int H, int W, int k, hipStream_t stream, float *logdet)
{
    if (!flow_split_supported(B, C, H, W, k))
        return INVCONV_ERR_VARIANT;
    const FlowParams fp{s, b, Q};
    if (C == 3 && k == 3) return launch_flow_fwd_split_ck<3, 3>(y, w, fp, z, B, H, W, stream, logdet);
    if (C == 3 && k == 5) return launch_flow_fwd_split_ck<3, 5>(y, w, fp, z, B, H, W, stream, logdet);
    if (C == 1 && k == 3) return launch_flow_fwd_split_ck<1, 3>(y, w, fp, z, B, H, W, stream, logdet);
    if (C == 2 && k == 3) return launch_flow_fwd_split_ck<2, 3>(y, w, fp, z, B, H, W, stream, logdet);
    if (C == 4 && k == 3) return launch_flow_fwd_split_ck<4, 3>(y, w, fp, z, B, H, W, stream, logdet);
    return INVCONV_ERR_VARIANT;
}

int launch_solve_wave_split(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W, int k,
                            hipStream_t stream, float *logdet)
{
    if (!wave_supported(C, H, k))
        return INVCONV_ERR_VARIANT;
    if (C == 3 && k == 3) return launch_wave_split_ck<3, 3>(dir, in, w, out, B, H, W, stream, logdet);
    if (C == 3 && k == 5) return launch_wave_split_ck<3, 5>(dir, in, w, out, B, H, W, stream, logdet);
    if (C == 3 && k == 7) return launch_wave_split_ck<3, 7>(dir, in, w, out, B, H, W, stream, logdet);
    if (C == 3 && k == 9) return launch_wave_split_ck<3, 9>(dir, in, w, out, B, H, W, stream, logdet);
    if (C == 3 && k == 11) return launch_wave_split_ck<3, 11>(dir, in, w, out, B, H, W, stream, logdet);
    if (C == 1 && k == 3) return launch_wave_split_ck<1, 3>(dir, in, w, out, B, H, W, stream, logdet);
    if (C == 2 && k == 3) return launch_wave_split_ck<2, 3>(dir, in, w, out, B, H, W, stream, logdet);
    if (C == 4 && k == 3) return launch_wave_split_ck<4, 3>(dir, in, w, out, B, H, W, stream, logdet);
    return INVCONV_ERR_VARIANT;
}

// What the multi-workgroup launch wants for this shape: logs and counters of up to 2048 workgroups at once
size_t wave_bands_ws_bytes(int B, int C, int H, int W, int k)
{
    if (!wave_bands_supported(C, H, W, k) || !wave_bands_multi_preferred(B, H, W, k))
        return 0;
    const size_t nb = (H + 63) / 64;
    const size_t most = 2048 / nb < 1 ? 1 : 2048 / nb;
    return ((size_t)B < most ? (size_t)B : most) * wave_bands_multi_ws_per_image(H, W, k);
}

int launch_solve_wave_bands(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W, int k,
                            hipStream_t stream, SolveWs ws)
{
    if (!wave_bands_supported(C, H, W, k))
        return INVCONV_ERR_VARIANT;
    const bool multi = wave_bands_multi_preferred(B, H, W, k);
    if (C == 3 && k == 3) return multi ? launch_wave_bands_multi_ck<3, 3>(dir, in, w, out, B, H, W, stream, ws)
                                  : launch_wave_bands_ck<3, 3>(dir, in, w, out, B, H, W, stream, ws.err);
    if (C == 3 && k == 2) return multi ? launch_wave_bands_multi_ck<3, 2>(dir, in, w, out, B, H, W, stream, ws)
                                  : launch_wave_bands_ck<3, 2>(dir, in, w, out, B, H, W, stream, ws.err);
    if (C == 3 && k == 5) return multi ? launch_wave_bands_multi_ck<3, 5>(dir, in, w, out, B, H, W, stream, ws)
                                  : launch_wave_bands_ck<3, 5>(dir, in, w, out, B, H, W, stream, ws.err);
    if (C == 1 && k == 3) return multi ? launch_wave_bands_multi_ck<1, 3>(dir, in, w, out, B, H, W, stream, ws)
                                  : launch_wave_bands_ck<1, 3>(dir, in, w, out, B, H, W, stream, ws.err);
    if (C == 2 && k == 3) return multi ? launch_wave_bands_multi_ck<2, 3>(dir, in, w, out, B, H, W, stream, ws)
                                  : launch_wave_bands_ck<2, 3>(dir, in, w, out, B, H, W, stream, ws.err);
    if (C == 4 && k == 3) return multi ? launch_wave_bands_multi_ck<4, 3>(dir, in, w, out, B, H, W, stream, ws)
                                  : launch_wave_bands_ck<4, 3>(dir, in, w, out, B, H, W, stream, ws.err);
    return INVCONV_ERR_VARIANT;
}

int launch_solve_wave(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W, int k,
                      hipStream_t stream, float *logdet)
{
    if (!wave_supported(C, H, k))
        return INVCONV_ERR_VARIANT;
    if (C == 3 && k == 3) return launch_wave_ck<3, 3>(dir, in, w, out, B, H, W, stream, logdet);
    if (C == 3 && k == 2) return launch_wave_ck<3, 2>(dir, in, w, out, B, H, W, stream, logdet);
    if (C == 3 && k == 5) return launch_wave_ck<3, 5>(dir, in, w, out, B, H, W, stream, logdet);
    if (C == 3 && k == 7) return launch_wave_ck<3, 7>(dir, in, w, out, B, H, W, stream, logdet);
    if (C == 3 && k == 9) return launch_wave_ck<3, 9>(dir, in, w, out, B, H, W, stream, logdet);
    if (C == 3 && k == 11) return launch_wave_ck<3, 11>(dir, in, w, out, B, H, W, stream, logdet);
    if (C == 1 && k == 3) return launch_wave_ck<1, 3>(dir, in, w, out, B, H, W, stream, logdet);
    if (C == 2 && k == 3) return launch_wave_ck<2, 3>(dir, in, w, out, B, H, W, stream, logdet);
    if (C == 4 && k == 3) return launch_wave_ck<4, 3>(dir, in, w, out, B, H, W, stream, logdet);
    return INVCONV_ERR_VARIANT;
}

// ---------------------------------------------------------------------------
// bf16 storage (activations as bf16 in memory, fp32 arithmetic): the LDS-tile kernels with the conversion
// on the way in and out.  Few channels, images that fit LDS, C*H*W a multiple of 4, 8-byte aligned tensors.
// ---------------------------------------------------------------------------
static bool wave_tile_bf16_ck(int C, int k) { return (C == 3 && (k == 3 || k == 5)) || ((C == 1 || C == 2 || C == 4) && k == 3); }

bool wave_tile_bf16_supported(int C, int H, int W, int k)
{
    return wave_tile_bf16_ck(C, k) && wave_supported(C, H, k) && (C * H * W) % 4 == 0 &&
           (size_t)C * H * W * sizeof(float) <= 64 * 1024 && bwd_wave_lds_bytes(C, H, W, k) <= kMaxLdsBytes;
}

template <int C, int K>
static int launch_tile_bf16_ck(int dir, const bf16_t *in, const float *w, bf16_t *out, int B, int H, int W,
                               hipStream_t stream)
{
    const size_t lds = (size_t)C * H * W * sizeof(float);
    const void *fn = dir ? reinterpret_cast<const void *>(&k_solve_wave_tile<C, K, 1, bf16_t>)
                         : reinterpret_cast<const void *>(&k_solve_wave_tile<C, K, 0, bf16_t>);
    if (!ensure_dynamic_lds(fn, lds))
        return INVCONV_ERR_UNSUPPORTED;
    if (dir)
        hipLaunchKernelGGL((k_solve_wave_tile<C, K, 1, bf16_t>), dim3(B), dim3(64), lds, stream, in, w, out, H, W,
                           (float *)nullptr);
    else
        hipLaunchKernelGGL((k_solve_wave_tile<C, K, 0, bf16_t>), dim3(B), dim3(64), lds, stream, in, w, out, H, W,
                           (float *)nullptr);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

int launch_solve_wave_tile_bf16(int dir, const void *in, const float *w, void *out, int B, int C, int H, int W, int k,
                                hipStream_t stream)
{
    if (!wave_tile_bf16_supported(C, H, W, k))
        return INVCONV_ERR_VARIANT;
    const bf16_t *i16 = static_cast<const bf16_t *>(in);
    bf16_t *o16 = static_cast<bf16_t *>(out);
    if (C == 3 && k == 3) return launch_tile_bf16_ck<3, 3>(dir, i16, w, o16, B, H, W, stream);
    if (C == 3 && k == 5) return launch_tile_bf16_ck<3, 5>(dir, i16, w, o16, B, H, W, stream);
    if (C == 1 && k == 3) return launch_tile_bf16_ck<1, 3>(dir, i16, w, o16, B, H, W, stream);
    if (C == 2 && k == 3) return launch_tile_bf16_ck<2, 3>(dir, i16, w, o16, B, H, W, stream);
    if (C == 4 && k == 3) return launch_tile_bf16_ck<4, 3>(dir, i16, w, o16, B, H, W, stream);
    return INVCONV_ERR_VARIANT;
}

template <int C, int K>
static int launch_bwd_tile_bf16_ck(const bf16_t *x, const float *w, const bf16_t *g, bf16_t *v, float *part, int B,
                                   int H, int W, hipStream_t stream)
{
    const size_t lds = bwd_wave_lds_bytes(C, H, W, K);
    if (!ensure_dynamic_lds(reinterpret_cast<const void *>(&k_bwd_wave<C, K, false, true, bf16_t>), lds))
        return INVCONV_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((k_bwd_wave<C, K, false, true, bf16_t>), dim3(B), dim3(256), lds, stream, x, w, g, v, part, H, W);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

// dL/dy (bf16) and the per-image partial sums of dL/dw (fp32, from the unrounded dL/dy) in one launch
int launch_bwd_wave_tile_bf16(const void *x, const float *w, const void *g, void *v, float *part, int B, int C, int H,
                              int W, int k, hipStream_t stream)
{
    if (!wave_tile_bf16_supported(C, H, W, k))
        return INVCONV_ERR_VARIANT;
    const bf16_t *x16 = static_cast<const bf16_t *>(x), *g16 = static_cast<const bf16_t *>(g);
    bf16_t *v16 = static_cast<bf16_t *>(v);
    if (C == 3 && k == 3) return launch_bwd_tile_bf16_ck<3, 3>(x16, w, g16, v16, part, B, H, W, stream);
    if (C == 3 && k == 5) return launch_bwd_tile_bf16_ck<3, 5>(x16, w, g16, v16, part, B, H, W, stream);
    if (C == 1 && k == 3) return launch_bwd_tile_bf16_ck<1, 3>(x16, w, g16, v16, part, B, H, W, stream);
    if (C == 2 && k == 3) return launch_bwd_tile_bf16_ck<2, 3>(x16, w, g16, v16, part, B, H, W, stream);
    if (C == 4 && k == 3) return launch_bwd_tile_bf16_ck<4, 3>(x16, w, g16, v16, part, B, H, W, stream);
    return INVCONV_ERR_VARIANT;
}

// Conversion passes for the shapes the tile kernels do not take
__global__ void k_bf16_to_f32(const bf16_t *__restrict__ in, float *__restrict__ out, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        out[i] = bf16_to_float(in[i]);
}

__global__ void k_f32_to_bf16(const float *__restrict__ in, bf16_t *__restrict__ out, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        out[i] = float_to_bf16(in[i]);
}

int launch_bf16_to_f32(const void *in, float *out, size_t n, hipStream_t stream)
{
    const unsigned grid = (unsigned)((n + 255) / 256 < 65536 ? (n + 255) / 256 : 65536);
    hipLaunchKernelGGL(k_bf16_to_f32, dim3(grid), dim3(256), 0, stream, static_cast<const bf16_t *>(in), out, n);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

int launch_f32_to_bf16(const float *in, void *out, size_t n, hipStream_t stream)
{
    const unsigned grid = (unsigned)((n + 255) / 256 < 65536 ? (n + 255) / 256 : 65536);
    hipLaunchKernelGGL(k_f32_to_bf16, dim3(grid), dim3(256), 0, stream, in, static_cast<bf16_t *>(out), n);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

}  // namespace invconv
