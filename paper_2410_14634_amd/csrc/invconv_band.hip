// Band-systolic wavefront solve for 5 to 16 channels (laid out for C = 8, 12 or 16) on the matrix
// cores (v_mfma_f32_16x16x4_f32).  gfx950 only.
//
// A wave owns a band of 16 image rows.  Lane (n, g) = (lane % 16, lane / 16)
// owns row n of the band and the channel group g: channels CG*g .. CG*g+CG-1
// with CG = C/4.  At step t the wave holds one anti-diagonal of its band (lane
// row n is at column c = t - n - band delay), exactly as in the few-channel
// wave kernel: own-row history in registers, one message per step from the row
// above (DPP row_shr:1 inside each 16-lane group; lane n = 0 takes the message
// of the band above from LDS).
//
// With folded weights the update of one anti-diagonal is a dense contraction
// out[o][pixel] += Cf_tap[o][i] * x_tap[i][pixel] over (tap, i): M = output
// channel, N = the 16 pixels of the band, K = 4 input channels per instruction,
// one from each lane group.  The operand layouts of the instruction line up with
// the ownership above: the B operand of lane (n, g) is its own history value of
// channel CG*g + jj, and the four result registers of lane (n, g) are output
// rows 4g .. 4g+3, i.e. its own channels (row 4g+3 is padding when CG = 3).
//
// An image taller than 16 rows uses one wave per band inside one workgroup.
// Band b runs kBandDelay steps behind the skew of band b-1, all waves meet at a
// barrier once per step, and the last row of a band hands its messages to the
// next band through a small LDS ring.
#include "invconv_common.h"
#include "invconv_launch.h"
#include "invconv_wave_inverse.h"
#include <type_traits>

namespace invconv {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// value of the same channel group one image row up (row 0 of the band receives 0)
__device__ __forceinline__ float from_row_above16(float v)
{
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x111 /* row_shr:1 */, 0xf, 0xf, true));
}

constexpr int kBandPF = 8;      // steps of load prefetch
constexpr int kBandDelay = 1;   // extra steps a band lags behind the band above
constexpr int kRing = 4;        // depth of the band-to-band message ring

// MAXT: the most threads a launch may have (512 for k = 3; the folded taps of larger kernels need the registers
// of a workgroup of at most four waves).
// PAD: the image has Cr < 4 CG channels (5-7, 9-11, 13-15).  The lanes' channel slots beyond Cr carry zero weights in
// both operand roles, read as zero and are never stored, so the solve is that of the Cr real channels; the folded
// weights are then laid out with row length Cr.
// LDSW: the C k^2 / 4 folded taps of a lane do not fit its registers (k = 9, 11; 16 channels at k = 7): they stay in
// LDS, negated, and every matrix instruction fetches its A operand from there (a fixed address per lane and tap).
// Lanes whose A row is padding read some valid row: their result rows are never used.
template <int CG, int K, int DIR, int MAXT = 512, bool PAD = false, bool LDSW = false>
__global__ __launch_bounds__(MAXT) void k_solve_band(const float *__restrict__ in, const float *__restrict__ w,
                                                    float *__restrict__ out, int H, int W, int NB, float *logdet,
                                                    int Cr)
{
    static_assert(!(PAD && LDSW), "taps in LDS go with channel counts the lanes are laid out for");
    constexpr int C = 4 * CG;
    const int Cs = PAD ? Cr : C;        // channels of the image = row length of the folded weights
    extern __shared__ float smem[];
    float *sL = smem;
    float *sLinv = sL + C * C;
    float *sCf = sLinv + C * C;
    float *sW = sCf + K * K * C * C;        // (staging copy of the runtime-C fold; the compile-time-C fold does without)
    float *sMsg = LDSW ? sW : sW + K * K * C * C;       // [NB][kRing][K][16 groups*4]  (a = 0 unused)

    const int tid = threadIdx.x;
    const int band = tid >> 6, lane = tid & 63;
    const int n = lane & 15, g = lane >> 4;
    const int row = band * 16 + n;
    const bool row_ok = row < H;
    const int rr = row_ok ? row : H - 1;
    const unsigned Wst = row_ok ? (unsigned)W : 0u;

    // addressing: uniform pointer per (channel of this lane's group) + per-lane 32-bit byte offset
    const size_t img = (size_t)blockIdx.x * Cs * H * W;
    const char *chan_src[CG];
    char *chan_dst[CG];
    bool ch_ok[CG];
#pragma unroll
    for (int jj = 0; jj < CG; ++jj) {
        ch_ok[jj] = !PAD || CG * g + jj < Cs;
        const int ch = ch_ok[jj] ? CG * g + jj : 0;
        const size_t cb = img + (size_t)(DIR ? Cs - 1 - ch : ch) * H * W;
        chan_src[jj] = reinterpret_cast<const char *>(in + cb);
        chan_dst[jj] = reinterpret_cast<char *>(out + cb);
    }
    constexpr int kStep = DIR ? -4 : 4;
    const int row0 = 4 * (DIR ? (H - 1 - rr) * W + (W - 1) : rr * W);
    const int rowlo = DIR ? row0 - 4 * (W - 1) : row0;
    const int rowhi = DIR ? row0 : row0 + 4 * (W - 1);
    auto clamp_row = [&](int off) -> unsigned { return (unsigned)(off < rowlo ? rowlo : (off > rowhi ? rowhi : off)); };
    auto ld = [&](int jj, unsigned off) -> float {
        const float v = *reinterpret_cast<const float *>(chan_src[jj] + off);
        return ch_ok[jj] ? v : 0.0f;
    };
    auto st = [&](int jj, unsigned off, float v) {
        if (ch_ok[jj])
            *reinterpret_cast<float *>(chan_dst[jj] + off) = v;
    };

    // Local step tau = t - t_first of this band: lane row n is at column c = tau - n.
    const int t_first = band * (16 + kBandDelay);

    // first batch of input loads, issued before the weight preparation
    float yb[kBandPF][CG];
#pragma unroll
    for (int u = 0; u < kBandPF; ++u) {
        const unsigned off = clamp_row(row0 + kStep * (u - n));
#pragma unroll
        for (int jj = 0; jj < CG; ++jj)
            yb[u][jj] = ld(jj, off);
    }

    if (PAD)
        fold_weights<DIR, 0>(w, Cs, K, sL, sLinv, sCf, sW);
    else
        fold_weights<DIR, C>(w, C, K, sL, sLinv, sCf, sW);
    for (int idx = tid; idx < NB * kRing * K * 64; idx += blockDim.x)
        sMsg[idx] = 0.0f;

    // A operands of this lane: output row m = lane%16 -> channel o(m) = CG*(m/4) + m%4 (padding if m%4 >= CG),
    // K slot g -> input channel CG*g + jj
    const int m = n;
    const bool m_ok = (m & 3) < CG && (!PAD || CG * (m >> 2) + (m & 3) < Cs);
    const int om = m_ok ? CG * (m >> 2) + (m & 3) : 0;
    float wA[LDSW ? 1 : K][LDSW ? 1 : K][CG], wLi[CG];
    if constexpr (!LDSW) {
#pragma unroll
        for (int a = 0; a < K; ++a)
#pragma unroll
            for (int db = 0; db < K; ++db)
#pragma unroll
                for (int jj = 0; jj < CG; ++jj) {
                    const int ii = ch_ok[jj] ? CG * g + jj : 0;
                    const float cf = sCf[((a * K + db) * Cs + om) * Cs + ii];
                    wA[a][db][jj] = m_ok && ch_ok[jj] ? -cf : 0.0f;
                }
    }
#pragma unroll
    for (int jj = 0; jj < CG; ++jj) {
        const float lv = sLinv[om * Cs + (ch_ok[jj] ? CG * g + jj : 0)];
        wLi[jj] = m_ok && ch_ok[jj] ? lv : 0.0f;
    }
    if constexpr (LDSW) {
        for (int idx = tid; idx < K * K * C * C; idx += blockDim.x)
            sCf[idx] = -sCf[idx];
    }
    // A operand of tap (a, db), K slot jj: a register, or this lane's entry of the negated taps in LDS
    const float *cfp = sCf + om * C + CG * g;
    auto tapw = [&](int a, int db, int jj) -> float {
        if constexpr (LDSW)
            return cfp[(a * K + db) * C * C + jj];
        else
            return wA[a][db][jj];
    };
    __syncthreads();        // ring zeroed, weights read (or negated in place)
    if (band >= NB) {
        // helper waves of a single-band launch: they only speed up the weight preparation; the last one of the
        // first workgroup also forms the log-determinant when the caller asked for it
        if (logdet && blockIdx.x == 0 && band == 3)
            wave_logdet_any(w, Cs, K, H, W, logdet);
        return;
    }

    float xh[CG][K];
    f32x4 T[K];
#pragma unroll
    for (int jj = 0; jj < CG; ++jj)
#pragma unroll
        for (int db = 0; db < K; ++db)
            xh[jj][db] = 0.0f;
#pragma unroll
    for (int a = 0; a < K; ++a)
        T[a] = f32x4{0.f, 0.f, 0.f, 0.f};

#pragma unroll
    for (int u = 0; u < kBandPF; ++u)
#pragma unroll
        for (int jj = 0; jj < CG; ++jj)
            asm volatile("" : "+v"(yb[u][jj]));

    int c = -n;
    int ldoff = row0 + kStep * (kBandPF - n);
    f32x4 own = f32x4{0.f, 0.f, 0.f, 0.f};
    {
        const bool in_row = (unsigned)c < (unsigned)W;
#pragma unroll
        for (int jj = 0; jj < CG; ++jj)
            own = __builtin_amdgcn_mfma_f32_16x16x4f32(wLi[jj], in_row ? yb[0][jj] : 0.0f, own, 0, 0, 0);
        const unsigned off = clamp_row(ldoff);
#pragma unroll
        for (int jj = 0; jj < CG; ++jj)
            yb[0][jj] = ld(jj, off);
        ldoff += kStep;
    }

    const bool first_row = (n == 0) && (band > 0);      // takes its messages from the band above
    const bool last_row = (n == 15) && (band + 1 < NB); // hands its messages to the band below
    const float *msg_in = sMsg + (size_t)(band > 0 ? band - 1 : 0) * kRing * K * 64 + g * 4;
    float *msg_out = sMsg + (size_t)band * kRing * K * 64 + g * 4;

    // Every wave passes the same number of barriers: t_first before its own steps,
    // ntau during them (the same for all bands), and the rest afterwards.
    const int ntau = (16 + W - 1 + kBandPF - 1) / kBandPF * kBandPF;
    if (NB > 1) {
        for (int t = 0; t < t_first; ++t)
            __syncthreads();
    }
    for (int tau0 = 0; tau0 < ntau; tau0 += kBandPF) {
#pragma unroll
        for (int u = 0; u < kBandPF; ++u) {
            const int t = t_first + tau0 + u;
            // messages handed over by the band above kBandDelay+1 steps ago (used by row 0 only)
            const float *mi = msg_in + ((t - 1 - kBandDelay) & (kRing - 1)) * K * 64;
            float mrow[K][CG];
#pragma unroll
            for (int a = 1; a < K; ++a)
#pragma unroll
                for (int j = 0; j < CG; ++j)
                    mrow[a][j] = mi[a * 64 + j];

            float xn[CG];
#pragma unroll
            for (int j = 0; j < CG; ++j) {
                const float up = from_row_above16(T[1][j]);
                xn[j] = own[j] + (first_row ? mrow[1][j] : up);
            }
            if ((unsigned)c < Wst) {
                const unsigned off = (unsigned)(row0 + kStep * c);
#pragma unroll
                for (int j = 0; j < CG; ++j)
                    st(j, off, xn[j]);
            }
#pragma unroll
            for (int jj = 0; jj < CG; ++jj)
                xh[jj][0] = xn[jj];
#pragma unroll
            for (int a = 1; a < K; ++a) {
                f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
                if (a + 1 < K) {
#pragma unroll
                    for (int j = 0; j < CG; ++j) {
                        const float up = from_row_above16(T[a + 1][j]);
                        acc[j] = first_row ? mrow[a + 1][j] : up;
                    }
                }
#pragma unroll
                for (int db = K - 1; db >= 0; --db)     // oldest column first: only db = 0 waits for this step\'s result
#pragma unroll
                    for (int jj = 0; jj < CG; ++jj)
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(tapw(a, db, jj), xh[jj][db], acc, 0, 0, 0);
                T[a] = acc;
            }
            if (last_row) {
                float *mo = msg_out + (t & (kRing - 1)) * K * 64;
#pragma unroll
                for (int a = 1; a < K; ++a)
#pragma unroll
                    for (int j = 0; j < CG; ++j)
                        mo[a * 64 + j] = T[a][j];
            }
#pragma unroll
            for (int jj = 0; jj < CG; ++jj)
#pragma unroll
                for (int db = K - 1; db >= 1; --db)
                    xh[jj][db] = xh[jj][db - 1];
            c += 1;
            {
                const int s = (u + 1) % kBandPF;
                const bool in_row = (unsigned)c < (unsigned)W;
                f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int jj = 0; jj < CG; ++jj)
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(wLi[jj], in_row ? yb[s][jj] : 0.0f, acc, 0, 0, 0);
#pragma unroll
                for (int db = K - 1; db >= 1; --db)
#pragma unroll
                    for (int jj = 0; jj < CG; ++jj)
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(tapw(0, db, jj), xh[jj][db], acc, 0, 0, 0);
                own = acc;
                const unsigned off = clamp_row(ldoff);
#pragma unroll
                for (int jj = 0; jj < CG; ++jj)
                    yb[s][jj] = ld(jj, off);
                ldoff += kStep;
            }
            if (NB > 1)
                __syncthreads();
        }
    }
    if (NB > 1) {
        const int rest = (NB - 1 - band) * (16 + kBandDelay);
        for (int t = 0; t < rest; ++t)
            __syncthreads();
        // (the first band is through with its barriers when the last band ends: it has time for the log-determinant)
        if (logdet && blockIdx.x == 0 && band == 0)
            wave_logdet_any(w, Cs, K, H, W, logdet);
    }
}

// ---------------------------------------------------------------------------
// Images of at most 16 rows (one band, k = 3): the 27 matrix instructions of a step are split over
// the four waves of the workgroup by the age of their input, so that the wave on the chain of
// dependent steps issues only the 9 that read the pixel just solved.  With x_s the diagonal solved
// at step s (lane (n, g) as above) and A[a][db] the folded taps,
//   T1_s = up(T2_{s-1}) + A[1][0] x_s + { A[1][1] x_{s-1} + A[1][2] x_{s-2} }        = T1p_s + F1_s
//   T2_s =                A[2][0] x_s + { A[2][1] x_{s-1} + A[2][2] x_{s-2} }        = T2p_s + G2_s
//   own_{s+1} =           A[0][1] x_s + { Linv y_{s+1}    + A[0][2] x_{s-1} }        = ownp_s + O_{s+1}
//   x_{s+1} = own_{s+1} + up(T1_s)
// The braces only need x_{s-1}: waves 1, 2 and 3 form F1_s, G2_s and O_{s+1} during step s (x_{s-1}
// was published through LDS before the barrier that ended step s-1) and wave 0 picks them up at the
// start of step s+1, after the barrier that ends step s.  Wave 0 forms T1p, T2p and ownp itself.
// Wave 1 also writes x to global memory, wave 3 reads y.  One barrier per step.
// ---------------------------------------------------------------------------
// MAP (forward direction): the kernel is the forward pass of a whole flow step (Section 4.1: then Actnorm a = s x + b
// and the 1 x 1 convolution z = Q a).  The wave that stores applies z = A x + d (A = Q diag(s), d = Q b) to the
// diagonal it is about to store with CG more matrix instructions - the shape of Linv y: own values in, own channels
// out - so x never leaves the workgroup; one extra workgroup (the last) only forms the step's log-determinant,
// with Q eliminated by one wave, while the others solve.
struct BandFlowParams {
    const float *s, *b, *Q;
};

template <int CG, int DIR, bool PAD = false, bool MAP = false>
__global__ __launch_bounds__(256) void k_solve_band_split(const float *__restrict__ in, const float *__restrict__ w,
                                                          float *__restrict__ out, int H, int W, float *logdet, int Cr,
                                                          BandFlowParams fp = BandFlowParams{})
{
    static_assert(!MAP || DIR == 0, "the channel map goes with the forward solve");
    constexpr int K = 3, C = 4 * CG;
    const int Cs = PAD ? Cr : C;        // channels of the image (PAD: fewer than the lanes' 4 CG slots, as in k_solve_band)
    extern __shared__ float smem[];
    if (MAP && blockIdx.x == gridDim.x - 1) {
        // log|det dz/dy| of one image = H W (sum log|s| + log|det Q| - sum log|w[c][c][K-1][K-1]|)    (Section 4)
        if (logdet && threadIdx.x < 64) {
            double la = flow_invert_regs(fp.Q, Cs, reinterpret_cast<double *>(smem));
            double acc = 0.0;
            const int c = threadIdx.x;
            if (c < Cs)
                acc = log(fabs((double)fp.s[c])) - log(fabs((double)w[((c * Cs + c) * K + (K - 1)) * K + (K - 1)]));
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1)
                acc += __shfl_xor(acc, m, 64);
            if (c == 0)
                logdet[0] = (float)((double)H * (double)W * (acc + la));
        }
        return;
    }
    float *sL = smem;
    float *sLinv = sL + C * C;
    float *sCf = sLinv + C * C;
    float *sW = sCf + K * K * C * C;
    float *sX = sW + K * K * C * C;                     // [2][CG][64]  x of the last two steps
    f32x4 *sM = reinterpret_cast<f32x4 *>(sX + 2 * CG * 64);   // [2][3][64]  F1, G2, O of the last two steps

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    const bool row_ok = n < H;
    const int rr = row_ok ? n : H - 1;
    const unsigned Wst = row_ok ? (unsigned)W : 0u;

    const size_t img = (size_t)blockIdx.x * Cs * H * W;
    const char *chan_src[CG];
    char *chan_dst[CG];
    bool ch_ok[CG];
#pragma unroll
    for (int jj = 0; jj < CG; ++jj) {
        ch_ok[jj] = !PAD || CG * g + jj < Cs;
        const int ch = ch_ok[jj] ? CG * g + jj : 0;
        const size_t cb = img + (size_t)(DIR ? Cs - 1 - ch : ch) * H * W;
        chan_src[jj] = reinterpret_cast<const char *>(in + cb);
        chan_dst[jj] = reinterpret_cast<char *>(out + cb);
    }
    constexpr int kStep = DIR ? -4 : 4;
    const int row0 = 4 * (DIR ? (H - 1 - rr) * W + (W - 1) : rr * W);
    const int rowlo = DIR ? row0 - 4 * (W - 1) : row0;
    const int rowhi = DIR ? row0 : row0 + 4 * (W - 1);
    auto clamp_row = [&](int off) -> unsigned { return (unsigned)(off < rowlo ? rowlo : (off > rowhi ? rowhi : off)); };
    auto ld = [&](int jj, unsigned off) -> float {
        const float v = *reinterpret_cast<const float *>(chan_src[jj] + off);
        return ch_ok[jj] ? v : 0.0f;
    };
    auto st = [&](int jj, unsigned off, float v) {
        if (ch_ok[jj])
            *reinterpret_cast<float *>(chan_dst[jj] + off) = v;
    };

    // wave 3 reads y: slot u holds the input of the steps congruent to u; first batch = steps 0 .. kBandPF-1,
    // issued before the weight preparation so that both latencies overlap.  The other waves run the same
    // instructions on one common address (no branch around a load, next to no work for the address unit).
    float yb[kBandPF][CG];
#pragma unroll
    for (int u = 0; u < kBandPF; ++u) {
        const unsigned off = wave == 3 ? clamp_row(row0 + kStep * (u - n)) : 0u;
#pragma unroll
        for (int jj = 0; jj < CG; ++jj) {
            const float v = *reinterpret_cast<const float *>((wave == 3 ? chan_src[jj] : chan_src[0]) + off);
            yb[u][jj] = ch_ok[jj] ? v : 0.0f;
        }
    }

    if (PAD)
        fold_weights<DIR, 0>(w, Cs, K, sL, sLinv, sCf, sW);
    else
        fold_weights<DIR, C>(w, C, K, sL, sLinv, sCf, sW);
    for (int idx = tid; idx < 2 * CG * 64 + 2 * 3 * 64 * 4; idx += 256)
        sX[idx] = 0.0f;

    const int m = n;
    const bool m_ok = (m & 3) < CG && (!PAD || CG * (m >> 2) + (m & 3) < Cs);
    const int om = m_ok ? CG * (m >> 2) + (m & 3) : 0;
    float wA[K][K][CG], wLi[CG];
#pragma unroll
    for (int a = 0; a < K; ++a)
#pragma unroll
        for (int db = 0; db < K; ++db)
#pragma unroll
            for (int jj = 0; jj < CG; ++jj) {
                const int ii = ch_ok[jj] ? CG * g + jj : 0;
                const float cf = sCf[((a * K + db) * Cs + om) * Cs + ii];
                wA[a][db][jj] = m_ok && ch_ok[jj] ? -cf : 0.0f;
            }
#pragma unroll
    for (int jj = 0; jj < CG; ++jj) {
        const float lv = sLinv[om * Cs + (ch_ok[jj] ? CG * g + jj : 0)];
        wLi[jj] = m_ok && ch_ok[jj] ? lv : 0.0f;
    }
    // the map's operands, laid out like wLi (row om, input channel CG g + jj), and its offset per own channel
    float wAz[MAP ? CG : 1], dz[MAP ? CG : 1];
    if (MAP && wave == 1) {     // (the storing wave)
#pragma unroll
        for (int jj = 0; jj < CG; ++jj) {
            const int ic = ch_ok[jj] ? CG * g + jj : 0;
            const float av = fp.Q[om * Cs + ic] * fp.s[ic];
            wAz[jj] = m_ok && ch_ok[jj] ? av : 0.0f;
            double acc = 0.0;
            for (int i = 0; i < Cs; ++i)
                acc += (double)fp.Q[ic * Cs + i] * (double)fp.b[i];
            dz[jj] = (float)acc;
        }
    }
    __syncthreads();

#pragma unroll
    for (int u = 0; u < kBandPF; ++u)
#pragma unroll
        for (int jj = 0; jj < CG; ++jj)
            asm volatile("" : "+v"(yb[u][jj]));

    // Step s = -1 only lets the helpers prepare O_0 = Linv y_0; the steps after the last diagonal only
    // let wave 1 store.  Every wave runs its own loop (so that no register state is merged across the
    // roles) over the same number of steps, one barrier each.
    const int nsteps = 16 + W - 1;
    const int total = nsteps + 2;       // steps -1 .. total-2, the same for every wave
    if (wave == 0) {
        f32x4 T1p = f32x4{0.f, 0.f, 0.f, 0.f}, T2p = T1p, ownp = T1p;
        for (int s = -1; s < total - 1; ++s) {
            const int rs = (s - 1) & 1;
            const f32x4 F1 = sM[(rs * 3 + 0) * 64 + lane], G2 = sM[(rs * 3 + 1) * 64 + lane],
                        O = sM[(rs * 3 + 2) * 64 + lane];
            const f32x4 T1 = T1p + F1, T2 = T2p + G2, own = ownp + O;
            float xn[CG];
#pragma unroll
            for (int j = 0; j < CG; ++j) {
                xn[j] = own[j] + from_row_above16(T1[j]);
                sX[((s & 1) * CG + j) * 64 + lane] = xn[j];
            }
            f32x4 a1 = f32x4{0.f, 0.f, 0.f, 0.f}, a2 = a1, a0 = a1;
#pragma unroll
            for (int j = 0; j < CG; ++j)
                a1[j] = from_row_above16(T2[j]);
#pragma unroll
            for (int jj = 0; jj < CG; ++jj) {
                a1 = __builtin_amdgcn_mfma_f32_16x16x4f32(wA[1][0][jj], xn[jj], a1, 0, 0, 0);
                a2 = __builtin_amdgcn_mfma_f32_16x16x4f32(wA[2][0][jj], xn[jj], a2, 0, 0, 0);
                a0 = __builtin_amdgcn_mfma_f32_16x16x4f32(wA[0][1][jj], xn[jj], a0, 0, 0, 0);
            }
            T1p = a1;
            T2p = a2;
            ownp = a0;
            __syncthreads();
        }
    } else if (wave == 1 || wave == 2) {
        // F1 (wave 1, a = 1) or G2 (wave 2, a = 2): A[a][1] x_{s-1} + A[a][2] x_{s-2}; wave 1 also stores x_{s-1}
        const int a = wave;
        float x1[CG], x2[CG], w1[CG], w2[CG];
#pragma unroll
        for (int jj = 0; jj < CG; ++jj) {
            x1[jj] = x2[jj] = 0.0f;
            w1[jj] = a == 1 ? wA[1][1][jj] : wA[2][1][jj];
            w2[jj] = a == 1 ? wA[1][2][jj] : wA[2][2][jj];
        }
        const unsigned Wst1 = a == 1 ? Wst : 0u;
        for (int s = -1; s < total - 1; ++s) {
#pragma unroll
            for (int jj = 0; jj < CG; ++jj) {
                x2[jj] = x1[jj];
                x1[jj] = sX[(((s - 1) & 1) * CG + jj) * 64 + lane];
            }
            f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f}, acc2 = acc;
#pragma unroll
            for (int jj = 0; jj < CG; ++jj) {
                acc2 = __builtin_amdgcn_mfma_f32_16x16x4f32(w2[jj], x2[jj], acc2, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(w1[jj], x1[jj], acc, 0, 0, 0);
            }
            sM[((s & 1) * 3 + (a - 1)) * 64 + lane] = acc + acc2;
            const int c = s - 1 - n;        // column of x_{s-1} in this lane's row
            if constexpr (MAP) {
                f32x4 zacc = f32x4{0.f, 0.f, 0.f, 0.f};
                if (a == 1) {
#pragma unroll
                    for (int jj = 0; jj < CG; ++jj)
                        zacc = __builtin_amdgcn_mfma_f32_16x16x4f32(wAz[jj], x1[jj], zacc, 0, 0, 0);
                }
                if ((unsigned)c < Wst1) {
                    const unsigned off = (unsigned)(row0 + kStep * c);
#pragma unroll
                    for (int j = 0; j < CG; ++j)
                        st(j, off, zacc[j] + dz[j]);
                }
            } else if ((unsigned)c < Wst1) {
                const unsigned off = (unsigned)(row0 + kStep * c);
#pragma unroll
                for (int j = 0; j < CG; ++j)
                    st(j, off, x1[j]);
            }
            __syncthreads();
        }
    } else {
        // O_{s+1} = Linv y_{s+1} + A[0][2] x_{s-1}
        float x1[CG];
        int ldoff = row0 + kStep * (kBandPF - n);       // unclamped offset of the next refill
        // one step; u = slot of the input of step s + 1 (s + 1 is congruent to u)
        auto step = [&](int s, int u, bool refill) {
#pragma unroll
            for (int jj = 0; jj < CG; ++jj)
                x1[jj] = sX[(((s - 1) & 1) * CG + jj) * 64 + lane];
            const bool in_row = (unsigned)(s + 1 - n) < (unsigned)W;
            f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f}, acc2 = acc;
#pragma unroll
            for (int jj = 0; jj < CG; ++jj) {
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(wLi[jj], in_row ? yb[u][jj] : 0.0f, acc, 0, 0, 0);
                acc2 = __builtin_amdgcn_mfma_f32_16x16x4f32(wA[0][2][jj], x1[jj], acc2, 0, 0, 0);
            }
            sM[((s & 1) * 3 + 2) * 64 + lane] = acc + acc2;
            if (refill) {       // the input of step s + 1 + kBandPF
                const unsigned off = clamp_row(ldoff);
#pragma unroll
                for (int jj = 0; jj < CG; ++jj)
                    yb[u][jj] = ld(jj, off);
                ldoff += kStep;
            }
            __syncthreads();
        };
        // whole blocks of kBandPF steps, then the rest without refills (its inputs are already there)
        const int nfull = total / kBandPF;
        int s0 = -1;
        for (int blk = 0; blk < nfull; ++blk, s0 += kBandPF) {
#pragma unroll
            for (int u = 0; u < kBandPF; ++u)
                step(s0 + u, u, true);
        }
        const int rest = total - nfull * kBandPF;
#pragma unroll
        for (int u = 0; u < kBandPF; ++u)
            if (u < rest)
                step(s0 + u, u, false);
    }
    if (!MAP && logdet && blockIdx.x == 0 && wave == 2)
        wave_logdet_any(w, Cs, K, H, W, logdet);
}

// ---------------------------------------------------------------------------
// Images of at most 16 rows with the larger kernels of the kernel-size ablation (k = 5, 7, 9, 11): the K K CG matrix
// instructions of a step split over NF + 2 waves by the age of their input, as the few-channel split solve does
// (lane = row there, lane (n, g) here).  With x_s the diagonal solved at step s and A[a][db] the folded taps,
//   T[a]_s    = up(T[a+1]_{s-1}) + A[a][0] x_s + { sum_{db>=1} A[a][db] x_{s-db} }   = Tp[a]_s + F[a]_s
//   own_{s+1} =                    A[0][1] x_s + { Linv y_{s+1} + sum_{db>=2} A[0][db] x_{s+1-db} }
//   x_{s+1}   = own_{s+1} + up(T[1]_s)
// The braces need nothing newer than x_{s-1}.  Wave 0, on the chain of dependent steps, publishes x_s through LDS
// and issues only the K CG instructions that read it; waves 1 .. NF form the F[a]_s of their rows a (delivered
// already shifted one row up), the last wave forms O_{s+1}, reads y and stores x.  Every role keeps only its own
// taps in registers, which is what lets k = 9 and 11 run from registers at all.  One barrier per step.
// ---------------------------------------------------------------------------
__host__ __device__ constexpr int band_splitk_nf(int K) { return K >= 7 ? (K - 1) / 2 : 2; }

template <int CG, int K>
__host__ __device__ constexpr size_t band_splitk_lds_floats()
{
    // Linv, folded taps, scratch L; x of the last two steps; messages of the last two steps (slot 0: O, slot a: F[a])
    return 2 * 16 * CG * CG + (size_t)K * K * 16 * CG * CG + 2 * CG * 64 + 2 * (size_t)K * 64 * 4;
}

template <int CG, int K, int DIR>
__global__ __launch_bounds__(64 * (band_splitk_nf(K) + 2)) void k_solve_band_splitk(const float *__restrict__ in,
                                                                                   const float *__restrict__ w,
                                                                                   float *__restrict__ out, int H,
                                                                                   int W, float *logdet)
{
    constexpr int C = 4 * CG, NF = band_splitk_nf(K), PER = (K - 1 + NF - 1) / NF, kOWave = NF + 1;
    extern __shared__ float smem[];
    float *sL = smem;
    float *sLinv = sL + C * C;
    float *sCf = sLinv + C * C;
    float *sX = sCf + K * K * C * C;                            // [2][CG][64]
    f32x4 *sM = reinterpret_cast<f32x4 *>(sX + 2 * CG * 64);    // [2][K][64]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    const bool row_ok = n < H;
    const int rr = row_ok ? n : H - 1;
    const unsigned Wst = row_ok ? (unsigned)W : 0u;

    const size_t img = (size_t)blockIdx.x * C * H * W;
    const char *chan_src[CG];
    char *chan_dst[CG];
#pragma unroll
    for (int jj = 0; jj < CG; ++jj) {
        const int ch = CG * g + jj;
        const size_t cb = img + (size_t)(DIR ? C - 1 - ch : ch) * H * W;
        chan_src[jj] = reinterpret_cast<const char *>(in + cb);
        chan_dst[jj] = reinterpret_cast<char *>(out + cb);
    }
    constexpr int kStep = DIR ? -4 : 4;
    const int row0 = 4 * (DIR ? (H - 1 - rr) * W + (W - 1) : rr * W);
    const int rowlo = DIR ? row0 - 4 * (W - 1) : row0;
    const int rowhi = DIR ? row0 : row0 + 4 * (W - 1);
    auto clamp_row = [&](int off) -> unsigned { return (unsigned)(off < rowlo ? rowlo : (off > rowhi ? rowhi : off)); };

    // the last wave reads y: slot u holds the input of the steps congruent to u (first batch before the weight
    // preparation; the other waves run the same instructions on one common address)
    float yb[kBandPF][CG];
#pragma unroll
    for (int u = 0; u < kBandPF; ++u) {
        const unsigned off = wave == kOWave ? clamp_row(row0 + kStep * (u - n)) : 0u;
#pragma unroll
        for (int jj = 0; jj < CG; ++jj)
            yb[u][jj] = *reinterpret_cast<const float *>((wave == kOWave ? chan_src[jj] : chan_src[0]) + off);
    }

    fold_weights<DIR, C>(w, C, K, sL, sLinv, sCf, sCf);         // (the compile-time-C fold needs no staging copy)
    for (int idx = tid; idx < 2 * CG * 64 + 2 * K * 64 * 4; idx += blockDim.x)
        sX[idx] = 0.0f;                                         // x and message slots are contiguous

    // A operands: row m = n -> output channel om (rows with m % 4 >= CG are padding: zero weights)
    const bool m_ok = (n & 3) < CG;
    const int om = m_ok ? CG * (n >> 2) + (n & 3) : 0;
    auto tap = [&](int a, int db, int jj) -> float {
        const float cf = sCf[((a * K + db) * C + om) * C + CG * g + jj];
        return m_ok ? -cf : 0.0f;
    };
#pragma unroll
    for (int u = 0; u < kBandPF; ++u)
#pragma unroll
        for (int jj = 0; jj < CG; ++jj)
            asm volatile("" : "+v"(yb[u][jj]));

    // step s = -1 only lets the last wave prepare O_0 = Linv y_0; the steps after the last diagonal only let it store
    const int nsteps = 16 + W - 1;
    const int total = nsteps + 2;       // steps -1 .. total-2, the same for every wave
    if (wave == 0) {
        float wC[K][CG];                // wC[a], a >= 1: A[a][0];  wC[0]: A[0][1]
#pragma unroll
        for (int a = 0; a < K; ++a)
#pragma unroll
            for (int jj = 0; jj < CG; ++jj)
                wC[a][jj] = a == 0 ? tap(0, 1, jj) : tap(a, 0, jj);
        __syncthreads();
        f32x4 Tp[K], ownp = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int a = 0; a < K; ++a)
            Tp[a] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int s = -1; s < total - 1; ++s) {
            const f32x4 *mi = sM + ((s - 1) & 1) * K * 64 + lane;
            f32x4 Fs[K];
#pragma unroll
            for (int a = 1; a < K; ++a)
                Fs[a] = mi[a * 64];
            const f32x4 own = ownp + mi[0];
            float xn[CG];
#pragma unroll
            for (int j = 0; j < CG; ++j) {
                xn[j] = own[j] + (from_row_above16(Tp[1][j]) + Fs[1][j]);
                sX[((s & 1) * CG + j) * 64 + lane] = xn[j];
            }
#pragma unroll
            for (int a = 1; a < K; ++a) {
                f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
                if (a + 1 < K) {
#pragma unroll
                    for (int j = 0; j < CG; ++j)
                        acc[j] = from_row_above16(Tp[a + 1][j]) + Fs[a + 1][j];
                }
#pragma unroll
                for (int jj = 0; jj < CG; ++jj)
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(wC[a][jj], xn[jj], acc, 0, 0, 0);
                Tp[a] = acc;
            }
            {
                f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int jj = 0; jj < CG; ++jj)
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(wC[0][jj], xn[jj], acc, 0, 0, 0);
                ownp = acc;
            }
            __syncthreads();
        }
    } else if (wave <= NF) {
        // F[a]_s = sum_{db>=1} A[a][db] x_{s-db} for this wave's rows a = A_LO .. A_LO + PER - 1
        const int a_lo = (wave - 1) * PER + 1;
        float wF[PER][K][CG];           // [.][db], db >= 1
#pragma unroll
        for (int q = 0; q < PER; ++q)
#pragma unroll
            for (int db = 1; db < K; ++db)
#pragma unroll
                for (int jj = 0; jj < CG; ++jj)
                    wF[q][db][jj] = a_lo + q < K ? tap(a_lo + q, db, jj) : 0.0f;
        __syncthreads();
        float xo[K][CG];                // xo[db] = x_{s-db}, db >= 1
#pragma unroll
        for (int db = 0; db < K; ++db)
#pragma unroll
            for (int jj = 0; jj < CG; ++jj)
                xo[db][jj] = 0.0f;
        for (int s = -1; s < total - 1; ++s) {
#pragma unroll
            for (int db = K - 1; db >= 2; --db)
#pragma unroll
                for (int jj = 0; jj < CG; ++jj)
                    xo[db][jj] = xo[db - 1][jj];
#pragma unroll
            for (int jj = 0; jj < CG; ++jj)
                xo[1][jj] = sX[(((s - 1) & 1) * CG + jj) * 64 + lane];
            f32x4 *mo = sM + (s & 1) * K * 64 + lane;
#pragma unroll
            for (int q = 0; q < PER; ++q) {
                f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f}, acc2 = acc;
#pragma unroll
                for (int db = K - 1; db >= 1; --db)
#pragma unroll
                    for (int jj = 0; jj < CG; ++jj) {
                        if ((db ^ jj) & 1)
                            acc2 = __builtin_amdgcn_mfma_f32_16x16x4f32(wF[q][db][jj], xo[db][jj], acc2, 0, 0, 0);
                        else
                            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(wF[q][db][jj], xo[db][jj], acc, 0, 0, 0);
                    }
                acc += acc2;
                f32x4 up = f32x4{0.f, 0.f, 0.f, 0.f};      // what the row below will add: F[a] of the row above
#pragma unroll
                for (int j = 0; j < CG; ++j)
                    up[j] = from_row_above16(acc[j]);
                if (a_lo + q < K)
                    mo[(a_lo + q) * 64] = up;
            }
            __syncthreads();
        }
    } else {
        // O_{s+1} = Linv y_{s+1} + sum_{db>=2} A[0][db] x_{s+1-db}; also x_{s-1} to global memory
        float wO[K][CG], wLi[CG];       // wO[db], db >= 2
#pragma unroll
        for (int db = 2; db < K; ++db)
#pragma unroll
            for (int jj = 0; jj < CG; ++jj)
                wO[db][jj] = tap(0, db, jj);
#pragma unroll
        for (int jj = 0; jj < CG; ++jj) {
            const float lv = sLinv[om * C + CG * g + jj];
            wLi[jj] = m_ok ? lv : 0.0f;
        }
        __syncthreads();
        float xo[K][CG];                // xo[db] = x_{s+1-db}, db >= 2
#pragma unroll
        for (int db = 0; db < K; ++db)
#pragma unroll
            for (int jj = 0; jj < CG; ++jj)
                xo[db][jj] = 0.0f;
        int ldoff = row0 + kStep * (kBandPF - n);       // unclamped offset of the next refill
        auto step = [&](int s, int u, bool refill) {
#pragma unroll
            for (int db = K - 1; db >= 3; --db)
#pragma unroll
                for (int jj = 0; jj < CG; ++jj)
                    xo[db][jj] = xo[db - 1][jj];
#pragma unroll
            for (int jj = 0; jj < CG; ++jj)
                xo[2][jj] = sX[(((s - 1) & 1) * CG + jj) * 64 + lane];
            const bool in_row = (unsigned)(s + 1 - n) < (unsigned)W;
            f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f}, acc2 = acc;
#pragma unroll
            for (int jj = 0; jj < CG; ++jj)
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(wLi[jj], in_row ? yb[u][jj] : 0.0f, acc, 0, 0, 0);
#pragma unroll
            for (int db = K - 1; db >= 2; --db)
#pragma unroll
                for (int jj = 0; jj < CG; ++jj)
                    acc2 = __builtin_amdgcn_mfma_f32_16x16x4f32(wO[db][jj], xo[db][jj], acc2, 0, 0, 0);
            sM[(s & 1) * K * 64 + lane] = acc + acc2;
            const int c = s - 1 - n;        // column of x_{s-1} = xo[2] in this lane's row
            if ((unsigned)c < Wst) {
                const unsigned off = (unsigned)(row0 + kStep * c);
#pragma unroll
                for (int j = 0; j < CG; ++j)
                    *reinterpret_cast<float *>(chan_dst[j] + off) = xo[2][j];
            }
            if (refill) {       // the input of step s + 1 + kBandPF
                const unsigned off = clamp_row(ldoff);
#pragma unroll
                for (int jj = 0; jj < CG; ++jj)
                    yb[u][jj] = *reinterpret_cast<const float *>(chan_src[jj] + off);
                ldoff += kStep;
            }
            __syncthreads();
        };
        const int nfull = total / kBandPF;
        int s0 = -1;
        for (int blk = 0; blk < nfull; ++blk, s0 += kBandPF) {
#pragma unroll
            for (int u = 0; u < kBandPF; ++u)
                step(s0 + u, u, true);
        }
        const int rest = total - nfull * kBandPF;
#pragma unroll
        for (int u = 0; u < kBandPF; ++u)
            if (u < rest)
                step(s0 + u, u, false);
    }
    if (logdet && blockIdx.x == 0 && wave == 1)
        wave_logdet_any(w, C, K, H, W, logdet);
}

// taps in LDS instead of registers: k = 9 and 11, and k = 7 at 16 channels
static bool band_taps_in_lds(int Cp, int k) { return k >= 9 || (k == 7 && Cp > 12); }

size_t solve_band_lds_bytes(int C, int k, int NB)
{
    const size_t copies = band_taps_in_lds(C, k) ? 1 : 2;      // (the staging copy only exists beside register taps)
    return sizeof(float) * (2 * (size_t)C * C + copies * (size_t)k * k * C * C + (size_t)NB * kRing * k * 64);
}

// k = 3: at most 8 bands = 512 threads.  Other kernel sizes of the paper's kernel-size ablation (2, 5; 7 up to 12
// channels) run on the general kernel with at most four bands: a lane then keeps C k^2 / 4 folded taps in registers
// (147 at 12 channels, k = 7).  k = 9 and 11 (and 7 at 16 channels) do not have the registers: their taps stay in
// LDS (8, 12 or 16 channels only).
// Channel counts between the sizes the lanes are laid out for (5-7, 9-11, 13-15) run the next size up with the
// surplus channel slots switched off.
bool band_supported(int C, int H, int k)
{
    if (C < 5 || C > 16)
        return false;
    if (k == 3)
        return H <= 128;
    const int Cp = (C + 3) / 4 * 4;
    const bool size_ok = k == 2 || k == 5 || k == 7 || k == 9 || k == 11;
    if (band_taps_in_lds(Cp, k) && C != Cp)
        return false;
    return size_ok && H <= 64 && solve_band_lds_bytes(Cp, k, (H + 15) / 16) <= kMaxLdsBytes;
}

template <int CG, int K, bool PAD>
static int launch_band_ck(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W,
                          hipStream_t stream, float *logdet)
{
    const int NB = (H + 15) / 16;
    if (NB == 1 && K == 3) {
        const size_t lds1 = sizeof(float) * (2 * (size_t)16 * CG * CG + 2 * (size_t)K * K * 16 * CG * CG +
                                             2 * CG * 64 + 2 * 3 * 64 * 4);
        if (dir)
            hipLaunchKernelGGL((k_solve_band_split<CG, 1, PAD>), dim3(B), dim3(256), lds1, stream, in, w, out, H, W,
                               logdet, C);
        else
            hipLaunchKernelGGL((k_solve_band_split<CG, 0, PAD>), dim3(B), dim3(256), lds1, stream, in, w, out, H, W,
                               logdet, C);
        return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
    }
    if constexpr (K >= 5 && !PAD) {
        // one band, a larger kernel: the step split over the waves by the age of its input
        const size_t ldsk = sizeof(float) * band_splitk_lds_floats<CG, K>();
        if (NB == 1 && ldsk <= kMaxLdsBytes) {
            const void *fnk = dir ? reinterpret_cast<const void *>(&k_solve_band_splitk<CG, K, 1>)
                                  : reinterpret_cast<const void *>(&k_solve_band_splitk<CG, K, 0>);
            if (!ensure_dynamic_lds(fnk, ldsk))
                return INVCONV_ERR_UNSUPPORTED;
            const dim3 blk(64 * (band_splitk_nf(K) + 2));
            if (dir)
                hipLaunchKernelGGL((k_solve_band_splitk<CG, K, 1>), dim3(B), blk, ldsk, stream, in, w, out, H, W, logdet);
            else
                hipLaunchKernelGGL((k_solve_band_splitk<CG, K, 0>), dim3(B), blk, ldsk, stream, in, w, out, H, W, logdet);
            return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
        }
    }
    const size_t lds = solve_band_lds_bytes(4 * CG, K, NB);
    constexpr int MAXT = K == 3 ? 512 : 256;
    // a single band gets three helper waves for the weight preparation (its loop has no barriers)
    const int threads = NB == 1 ? 256 : 64 * NB;
    if (threads > MAXT)
        return INVCONV_ERR_VARIANT;
    constexpr bool LDSW = K >= 9 || (K == 7 && CG == 4);
    if constexpr (LDSW && PAD) {
        return INVCONV_ERR_VARIANT;
    } else {
        const void *fn = dir ? reinterpret_cast<const void *>(&k_solve_band<CG, K, 1, MAXT, PAD, LDSW>)
                             : reinterpret_cast<const void *>(&k_solve_band<CG, K, 0, MAXT, PAD, LDSW>);
        if (!ensure_dynamic_lds(fn, lds))
            return INVCONV_ERR_UNSUPPORTED;
        if (dir)
            hipLaunchKernelGGL((k_solve_band<CG, K, 1, MAXT, PAD, LDSW>), dim3(B), dim3(threads), lds, stream, in, w,
                               out, H, W, NB, logdet, C);
        else
            hipLaunchKernelGGL((k_solve_band<CG, K, 0, MAXT, PAD, LDSW>), dim3(B), dim3(threads), lds, stream, in, w,
                               out, H, W, NB, logdet, C);
        return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
    }
}

// Forward pass of a whole flow step on the one-band kernel: 5-16 channels, k = 3, images of at most 16 rows.
bool flow_band_supported(int C, int H, int k) { return k == 3 && H <= 16 && band_supported(C, H, k); }

template <int CG, bool PAD>
static int launch_flow_band_cg(const float *y, const float *w, BandFlowParams fp, float *z, int B, int C, int H, int W,
                               hipStream_t stream, float *logdet)
{
    constexpr int K = 3;
    const size_t lds1 = sizeof(float) * (2 * (size_t)16 * CG * CG + 2 * (size_t)K * K * 16 * CG * CG +
                                         2 * CG * 64 + 2 * 3 * 64 * 4);
    hipLaunchKernelGGL((k_solve_band_split<CG, 0, PAD, true>), dim3(B + 1), dim3(256), lds1, stream, y, w, z, H, W,
                       logdet, C, fp);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

int launch_flow_fwd_band(const float *y, const float *w, const float *s, const float *b, const float *Q, float *z,
                         int B, int C, int H, int W, int k, hipStream_t stream, float *logdet)
{
    if (!flow_band_supported(C, H, k))
        return INVCONV_ERR_VARIANT;
    const BandFlowParams fp{s, b, Q};
    auto by_cg = [&](auto pad_tag) -> int {
        constexpr bool PAD = decltype(pad_tag)::value;
        if (C <= 8) return launch_flow_band_cg<2, PAD>(y, w, fp, z, B, C, H, W, stream, logdet);
        if (C <= 12) return launch_flow_band_cg<3, PAD>(y, w, fp, z, B, C, H, W, stream, logdet);
        return launch_flow_band_cg<4, PAD>(y, w, fp, z, B, C, H, W, stream, logdet);
    };
    return C % 4 ? by_cg(std::true_type()) : by_cg(std::false_type());
}

int launch_solve_band(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W, int k,
                      hipStream_t stream, float *logdet)
{
    if (!band_supported(C, H, k))
        return INVCONV_ERR_VARIANT;
    auto by_k = [&](auto cg_tag, auto pad_tag) -> int {
        constexpr int CG = decltype(cg_tag)::value;
        constexpr bool PAD = decltype(pad_tag)::value;
        if (k == 3) return launch_band_ck<CG, 3, PAD>(dir, in, w, out, B, C, H, W, stream, logdet);
        if (k == 2) return launch_band_ck<CG, 2, PAD>(dir, in, w, out, B, C, H, W, stream, logdet);
        if (k == 5) return launch_band_ck<CG, 5, PAD>(dir, in, w, out, B, C, H, W, stream, logdet);
        if (k == 7) return launch_band_ck<CG, 7, PAD>(dir, in, w, out, B, C, H, W, stream, logdet);
        if (k == 9) return launch_band_ck<CG, 9, PAD>(dir, in, w, out, B, C, H, W, stream, logdet);
        if (k == 11) return launch_band_ck<CG, 11, PAD>(dir, in, w, out, B, C, H, W, stream, logdet);
        return INVCONV_ERR_VARIANT;
    };
    auto by_cg = [&](auto pad_tag) -> int {
        if (C <= 8) return by_k(std::integral_constant<int, 2>(), pad_tag);
        if (C <= 12) return by_k(std::integral_constant<int, 3>(), pad_tag);
        return by_k(std::integral_constant<int, 4>(), pad_tag);
    };
    return C % 4 ? by_cg(std::true_type()) : by_cg(std::false_type());
}

}  // namespace invconv
