// The single-wave systolic solve of few-channel images (C <= 4), shared by the kernel files that build on
// it: lane = image row, the wave holds one anti-diagonal, neighbours travel through DPP shifts.  gfx950 only.
#pragma once
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

// value of the lane above; lane 0 keeps `first` (what the row above the wave's first row sent)
__device__ __forceinline__ float from_lane_above_or(float first, float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, first),
                                                                 __builtin_bit_cast(int, v), 0x138 /* wave_shr:1 */,
                                                                 0xf, 0xf, false));
}

constexpr int kWavePF = 16;   // steps of load prefetch

// Weight preparation in registers, by every lane for itself (the kernel reads w
// with uniform addresses only): Linv = inverse of the lower-triangular
// current-pixel block; the lane keeps row o = lane%4 of it (zeros for o >= C) and
// folds it into every other tap.  MFMA A operands of this lane:
//   wLi[j] = Linv[o][j],   wA[a][db][i] = -(Linv W_tap)[o][i] for tap (a,db) up/left.
template <int C, int K, int DIR>
__device__ __forceinline__ void wave_fold_regs(const float *__restrict__ w, int o_lane, float (&wA)[K][K][C],
                                               float (&wLi)[C])
{
    float Lm[C][C], Li[C][C], rd[C];
#pragma unroll
    for (int o = 0; o < C; ++o)
#pragma unroll
        for (int i = 0; i < C; ++i)
            Lm[o][i] = weff<DIR>(w, C, K, o, i, K - 1, K - 1);
#pragma unroll
    for (int o = 0; o < C; ++o)
        rd[o] = 1.0f / Lm[o][o];
#pragma unroll
    for (int j = 0; j < C; ++j) {
#pragma unroll
        for (int o = 0; o < C; ++o) {
            if (o < j) {
                Li[o][j] = 0.0f;
            } else if (o == j) {
                Li[o][j] = rd[j];
            } else {
                float sum = 0.0f;
#pragma unroll
                for (int m = j; m < o; ++m)
                    sum += Lm[o][m] * Li[m][j];
                Li[o][j] = -sum * rd[o];
            }
        }
    }
#pragma unroll
    for (int j = 0; j < C; ++j) {
        float v = 0.0f;
#pragma unroll
        for (int o = 0; o < C; ++o)
            v = (o_lane == o) ? Li[o][j] : v;
        wLi[j] = v;
    }
#pragma unroll
    for (int a = 0; a < K; ++a)
#pragma unroll
        for (int db = 0; db < K; ++db)
#pragma unroll
            for (int i = 0; i < C; ++i) {
                float sum = 0.0f;
                if (a != 0 || db != 0) {
#pragma unroll
                    for (int j = 0; j < C; ++j)
                        sum += wLi[j] * weff<DIR>(w, C, K, j, i, K - 1 - a, K - 1 - db);
                }
                wA[a][db][i] = -sum;
            }
}


// Images of more than 64 rows are cut into bands of 64 rows, one wave each, all in one workgroup
// (BANDS).  A band is the single-wave solve on its own rows and its own clock (local step j,
// lane l at column j - l); what row 63 of the band above would have handed to lane 0 through the
// DPP shift arrives through LDS instead: after its local step j' the upper band's lane 63 appends
// its messages T[1..K-1] to a log, entry j'; the lower band's lane 0 needs entry j + 63 at its step
// j (its row is 64 rows further down, so the same anti-diagonal is 64 local steps earlier).  The
// log keeps every step (no slot is reused, so a fast upper band can never overwrite what the
// lower one has not read), progress is published once per block of kWavePF steps in an LDS
// counter, and the lower band starts a block only when the counter covers the block's last entry.
// The upper band never waits for the lower one, so the waits end; they are bounded all the same.
struct WaveBands {
    int band;           // this wave's band
    int nbands;
    const f32x4 *log_in;    // [log_steps][K - 1]: what the band above sent (valid offset also for band 0)
    f32x4 *log_out;         // [log_steps][K - 1]: what this band sends (valid offset also for the last band)
    const int *prog_in;     // local steps of the band above whose entries are in log_in
    int *prog_out;          // local steps of this band whose entries are in log_out
    int log_steps;      // entries per band, a multiple of kWavePF
    f32x4 *scratch;     // [64][K - 1] write-only dump for the lanes that have nothing to send
    int spin_limit;     // polls of prog_in before a waiting band gives up
    int *err;           // device error word (may be null): set to 1 when a wait ran out
    // solve_wave_ring_body only: the band's rows pass through an LDS ring that other waves fill and drain
    float *ring;            // [C][64 rows][kRingStride], solve coordinates, column c at c % kRingCols
    const int *io_loaded;   // load blocks in the ring, counted from block -1: block j may start at j + 2
    int *io_done;           // blocks this wave has finished
    int *io_lost;           // set when a wave of the workgroup gave up a wait: the draining wave then writes NaN
};

// Columns of a row the ring holds (four chunks of kWavePF columns), and the distance between rows.  Lane r
// reads column t - r at step t: word r * kRingStride + t - r, bank (3r + t) % 32, distinct over the 32 lanes
// of either half of the wave (LDS has 32 banks of 4 bytes and serves a 64-lane access as two halves);
// the 16-byte accesses of the filling and draining waves (16 rows, same columns) spread over all banks too.
constexpr int kRingCols = 64;
constexpr int kRingStride = 68;

// Row r of a band needs, in block j (steps 16j .. 16j+15, and the input of step 16j+16 for the look-ahead
// of `own`), columns 16j-r .. 16j+16-r.  With rho(r) = floor((r-1)/16) these fall into chunks j-rho-1 and
// j-rho, so the input of block j is complete once every row has chunk j-rho(r): "load block j".
__device__ __forceinline__ int ring_rho(int r) { return (r - 1) >> 4; }

// Body of the solve for image n, executed by one full wave (lanes 0..63 of the
// calling workgroup).  With LDS_COPY the result is also written to lds_copy as a
// [C][H][W] tile in image (not mirrored) coordinates.
// With TILE the image lives in lds_copy (input on entry, result on return) and global memory is not touched.
// With PACK (TILE only, H <= 32) the wave solves two images at once, lanes 0..31 the rows of the one at
// lds_copy and lanes 32..63 the rows of the one pack_stride floats behind it (pack_second: that image
// exists); lane 32, a first row, takes nothing from lane 31.
template <int C, int K, int DIR, bool LDS_COPY, bool BANDS = false, bool TILE = false, bool PACK = false>
__device__ __forceinline__ void solve_wave_body(const float *__restrict__ in, const float *__restrict__ w,
                                                float *__restrict__ out, int H, int W, int n, float *lds_copy,
                                                WaveBands wb = WaveBands{}, bool pack_second = false,
                                                int pack_stride = 0)
{
    static_assert(!PACK || (TILE && !BANDS), "two images per wave only on LDS tiles");
    static_assert(C >= 1 && C <= 4, "one 4-row MFMA block per pixel");
    // All 64 lanes stay active to the end: the matrix instruction reads its weight
    // operand from every lane of a 4-lane block, whatever the execution mask says.
    // Lanes past the last row compute on clamped inputs and never store.
    const int lane = threadIdx.x & 63;
    const int r = PACK ? lane & 31 : lane;            // row inside the band (lane, or lane within its half)
    const bool second = PACK && lane >= 32;
    const bool top = PACK && r == 0;                  // a first row: nothing arrives from the lane above
    const int grow = BANDS ? 64 * wb.band + r : r;    // image row
    const bool row_ok = grow < H && (!second || pack_second);
    const int rr = grow < H ? grow : H - 1;
    const int o_lane = lane & 3;
    auto from_above = [&](float v) -> float {
        const float m = from_lane_above(v);
        return PACK ? (top ? 0.0f : m) : m;
    };
    const unsigned Wst = row_ok ? (unsigned)W : 0u;   // columns this lane may store

    // Element (ch, r, c) of this image, in solve coordinates, sits at
    // chan[ch] (uniform pointer) + rowoff (per lane) +- 4c bytes: one 32-bit lane
    // offset serves all channels, the addressing form global loads take directly.
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
    constexpr int kStep = DIR ? -4 : 4;               // bytes per column in solve order
    const int row0 = 4 * ((DIR ? (H - 1 - rr) * W + (W - 1) : rr * W) + (second ? pack_stride : 0));   // byte offset of column 0
    // Lowest / highest byte offset a load may use: the ends of the row in global memory.  On an LDS tile
    // the ends of the channel plane instead: a lane outside its row then reads some other row's element at
    // row0 + 4 (t - r), an address whose bank differs from lane to lane like those of the lanes inside,
    // whereas offsets clamped to the row ends (row * W: one bank when W is a multiple of 32) made
    // every read a many-way bank conflict for as long as part of the wave was outside the image.
    const int plane0 = 4 * (second ? pack_stride : 0);
    const int rowlo = TILE ? plane0 : (DIR ? row0 - 4 * (W - 1) : row0);
    const int rowhi = TILE ? plane0 + 4 * (H * W - 1) : (DIR ? row0 : row0 + 4 * (W - 1));
    auto clamp_row = [&](int off) -> unsigned { return (unsigned)(off < rowlo ? rowlo : (off > rowhi ? rowhi : off)); };
    auto ld = [&](int ch, unsigned off) -> float {
        return *reinterpret_cast<const float *>((TILE ? chan_lds[ch] : chan_src[ch]) + off);
    };
    // A band whose bounded wait for the band above ran out has no valid input any more: from then on it
    // stores NaN instead of results, so that a lost hand-over can never pass for a solution.
    bool lost = false;
    auto st = [&](int ch, unsigned off, float v) {
        if (BANDS)
            v = lost ? __builtin_nanf("") : v;
        if (!TILE)
            *reinterpret_cast<float *>(chan_dst[ch] + off) = v;
        if (LDS_COPY || TILE)
            *reinterpret_cast<float *>(chan_lds[ch] + off) = v;
    };

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

    float wA[K][K][C], wLi[C];
    wave_fold_regs<C, K, DIR>(w, o_lane, wA, wLi);

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

    const int band_rows = BANDS ? (H - 64 * wb.band < 64 ? H - 64 * wb.band : 64) : H;
    const int nsteps = band_rows + W - 1;
    const bool recv = BANDS && wb.band > 0, send = BANDS && wb.band + 1 < wb.nbands;
    // (plain offsets from the LDS base, never a null alternative: the accesses stay LDS instructions)
    const f32x4 *log_in = wb.log_in;
    f32x4 *log_out = wb.log_out;
    f32x4 M[K];          // M[a]: what the band above sent for this step (used by lane 0 only)
#pragma unroll
    for (int a = 0; a < K; ++a)
        M[a] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int t0 = 0; t0 < nsteps; t0 += kWavePF) {
        if (recv && !lost) {
            // entries t0 + 63 .. t0 + 63 + kWavePF - 1 of the upper band's log are needed
            int need = t0 + 64 + kWavePF;
            need = need > wb.log_steps ? wb.log_steps : need;
            int spins = 0;
            while (__hip_atomic_load(wb.prog_in, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < need &&
                   ++spins < wb.spin_limit)
                __builtin_amdgcn_s_sleep(1);
            if (__hip_atomic_load(wb.prog_in, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < need) {
                lost = true;        // the wait ran out: carry on (every wave still finishes), results are NaN
                if (wb.err && r == 0)
                    __hip_atomic_store(wb.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        // Entry of the first step now, the others one step ahead of their use (volatile: the read is
        // issued where it is written, well before the value is needed).
        f32x4 Mn[K];
        if (recv) {
            const int e = t0 + 63 < wb.log_steps ? t0 + 63 : wb.log_steps - 1;
#pragma unroll
            for (int a = 1; a < K; ++a)
                M[a] = log_in[e * (K - 1) + a - 1];
        }
#pragma unroll
        for (int u = 0; u < kWavePF; ++u) {
            if (recv && u + 1 < kWavePF) {
                int e = t0 + u + 64;
                e = e < wb.log_steps ? e : wb.log_steps - 1;     // past the upper band's last step: unused
#pragma unroll
                for (int a = 1; a < K; ++a)
                    Mn[a] = *(const volatile __attribute__((address_space(3))) f32x4 *)(log_in + e * (K - 1) + a - 1);
            }
            // x(r,c) = own + (message from the row above, computed there one step ago)
            float xn[C];
#pragma unroll
            for (int o = 0; o < C; ++o)
                xn[o] = own[o] + (BANDS ? from_lane_above_or(M[1][o], T[1][o]) : from_above(T[1][o]));
            if (BANDS) {        // after a lost wait NaN also travels on to the rows and bands below
#pragma unroll
                for (int o = 0; o < C; ++o)
                    xn[o] = lost ? __builtin_nanf("") : xn[o];
            }
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
                        acc[o] = BANDS ? from_lane_above_or(M[a + 1][o], T[a + 1][o]) : from_above(T[a + 1][o]);
                }
#pragma unroll
                for (int db = K - 1; db >= 0; --db)     // oldest column first: only db = 0 waits for this step's result
#pragma unroll
                    for (int i = 0; i < C; ++i)
                        acc = __builtin_amdgcn_mfma_f32_4x4x1f32(wA[a][db][i], xh[i][db], acc, 0, 0, 0);
                T[a] = acc;
            }
            if (send) {
                // lane 63 appends to the log; the other lanes write to a scratch line of their own, so that
                // no branch surrounds the LDS write (a branch makes the wait counters conservative)
                f32x4 *dst = r == 63 ? log_out + (t0 + u) * (K - 1) : wb.scratch + r * (K - 1);
#pragma unroll
                for (int a = 1; a < K; ++a)
                    dst[a - 1] = T[a];
            }
            if (recv && u + 1 < kWavePF) {
#pragma unroll
                for (int a = 1; a < K; ++a)
                    M[a] = Mn[a];
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
                for (int db = K - 1; db >= 1; --db)
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
        if (send)       // the block's log entries are written (LDS operations of a wave complete in order)
            __hip_atomic_store(wb.prog_out, t0 + kWavePF, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
}

// The band solve with input and result in the LDS ring of its workgroup (wb.ring): the same recurrence as
// solve_wave_body with BANDS, written for a wave whose step is bound by the number of instructions it
// issues (a 64-lane vector instruction occupies the issue port for four clocks): a step touches LDS in ONE
// batch of instructions right after the pixel is known - result into the ring (in place of its input), the
// previous step's messages into the outgoing log, the input two steps ahead out of the ring, the incoming
// log entry of the next step - followed by the matrix instructions of the step.  What the batch fetched is
// first used a whole step later, so the one wait per step (LDS operations complete in order) finds
// everything done.  Nothing in a step depends on a wave-uniform condition: every band receives (the first
// band's incoming log is zeros and complete) and sends (the last band's log goes nowhere).
// Another wave has put the input of block j into the ring before io_loaded reaches j + 2; io_done tells the
// draining wave which blocks are complete.  Entry e of the outgoing log is written at step e + 1 and
// published with the step after that.  Global memory is not touched.  DIR only selects the weights: the
// filling and draining waves do the mirroring.
// (Tried: splitting every chain of products into the part that needs the current pixel and the part that
// does not, the latter issued a step ahead - the extra register moves cost more issue slots than the
// shorter dependent chain saves: 163 us against 152 us for one 3x256x256 image.)
template <int C, int K, int DIR>
__device__ __forceinline__ void solve_wave_ring_body(const float *__restrict__ w, int H, int W, WaveBands wb)
{
    static_assert(C >= 1 && C <= 4, "one 4-row MFMA block per pixel");
    const int r = threadIdx.x & 63;
    const bool row_ok = 64 * wb.band + r < H;
    const unsigned Wst = row_ok ? (unsigned)W : 0u;
    const int band_rows = H - 64 * wb.band < 64 ? H - 64 * wb.band : 64;
    const int nblocks = (band_rows + W - 1 + kWavePF - 1) / kWavePF;

    char *ringb = reinterpret_cast<char *>(wb.ring) + r * kRingStride * 4;
    constexpr unsigned kPlane = 64 * kRingStride * 4;
    auto ring_at = [&](int step) -> char * { return ringb + (((step - r) & (kRingCols - 1)) << 2); };
    char *dump = reinterpret_cast<char *>(wb.scratch + r * (K - 1));     // 16 (K - 1) bytes nobody reads
    const f32x4 *log_in = wb.log_in;
    f32x4 *log_out = wb.log_out;

    const f32x4 nan4 = f32x4{__builtin_nanf(""), __builtin_nanf(""), __builtin_nanf(""), __builtin_nanf("")};
    f32x4 own = f32x4{0.f, 0.f, 0.f, 0.f};
    bool lost = false;
    // A wait that ran out: carry on without waiting (every wave still finishes), and from here on everything
    // is NaN - put into `own` it spreads to the results, to the rows below and to the bands below by itself.
    auto give_up = [&]() {
        lost = true;
        __hip_atomic_store(wb.io_lost, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (wb.err && r == 0)
            __hip_atomic_store(wb.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };
    auto wait_for = [&](const int *counter, int need) {
        if (lost)
            return;
        int spins = 0;
        while (__hip_atomic_load(counter, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < need &&
               ++spins < wb.spin_limit)
            __builtin_amdgcn_s_sleep(1);
        if (__hip_atomic_load(counter, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < need)
            give_up();
    };

    float wA[K][K][C], wLi[C];
    wave_fold_regs<C, K, DIR>(w, r & 3, wA, wLi);

    float xh[C][K];      // xh[i][db] = x(r, c-db)
    f32x4 T[K];          // T[a], a >= 1: message for pixel (r+a, c), negated sums (of the previous step)
    f32x4 Mn[K];         // incoming log entry of the coming step (lane 0 uses it)
    float yb[2][C];      // input of step t at slot t & 1, fetched two steps ahead
#pragma unroll
    for (int i = 0; i < C; ++i)
#pragma unroll
        for (int db = 0; db < K; ++db)
            xh[i][db] = 0.0f;
#pragma unroll
    for (int a = 0; a < K; ++a) {
        T[a] = f32x4{0.f, 0.f, 0.f, 0.f};
        Mn[a] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // own = Linv y - (own-row taps) of the coming pixel, prepared one step ahead
    wait_for(wb.io_loaded, 2);
    wait_for(wb.prog_in, 64 + kWavePF < wb.log_steps ? 64 + kWavePF : wb.log_steps);
    {
        const bool in_row = r == 0;                  // column -r at step 0
#pragma unroll
        for (int j = 0; j < C; ++j) {
            const float y0 = *reinterpret_cast<const float *>(ring_at(0) + j * kPlane);
            own = __builtin_amdgcn_mfma_f32_4x4x1f32(wLi[j], in_row ? y0 : 0.0f, own, 0, 0, 0);
        }
        const int e = 63 < wb.log_steps ? 63 : wb.log_steps - 1;
#pragma unroll
        for (int a = 1; a < K; ++a)
            Mn[a] = log_in[e * (K - 1) + a - 1];
    }

    for (int j = 0; j < nblocks; ++j) {
        const int t0 = j * kWavePF;
        if (j > 0) {
            wait_for(wb.io_loaded, j + 2);
            const int need = t0 + 64 + kWavePF;      // entries below t0 + 80: the last one serves step t0 + 16
            wait_for(wb.prog_in, need < wb.log_steps ? need : wb.log_steps);
        }
        if (lost)
            own = nan4;
        // the read-ahead never crosses into the next block's input, so step t0 + 1 is fetched here
#pragma unroll
        for (int ch = 0; ch < C; ++ch)
            yb[1][ch] = *reinterpret_cast<const float *>(ring_at(t0 + 1) + ch * kPlane);
#pragma unroll
        for (int u = 0; u < kWavePF; ++u) {
            const int t = t0 + u;
            // ---- the pixel: x(r, c) = own + (message from the row above, computed there one step ago)
            f32x4 M[K];
#pragma unroll
            for (int a = 1; a < K; ++a) {
                // (all four registers of an entry stay reserved until here, also the unused ones of C < 4:
                // a register handed out again while its load is in flight would make the wave wait for it)
                asm volatile("" : "+v"(Mn[a]));
                M[a] = Mn[a];
            }
            if (u == 1)     // entries below t0 were written with step t0 at the latest, and step t0 is complete
                __hip_atomic_store(wb.prog_out, t0, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
            float xn[C];
#pragma unroll
            for (int o = 0; o < C; ++o)
                xn[o] = own[o] + from_lane_above_or(M[1][o], T[1][o]);
            __builtin_amdgcn_sched_barrier(0);
            // ---- the LDS batch of the step
            {
                // (lanes with nothing to store write to a dump slot of their own: a branch around a store
                // costs more issue slots than the select of an address)
                const bool valid = (unsigned)(t - r) < Wst;
                char *dst = valid ? ring_at(t) : dump;
                const unsigned cstep = valid ? kPlane : 4u;
#pragma unroll
                for (int o = 0; o < C; ++o)
                    *reinterpret_cast<float *>(dst + o * cstep) = xn[o];
                f32x4 *ldst = (r == 63 && t > 0) ? log_out + (t - 1) * (K - 1) : reinterpret_cast<f32x4 *>(dump);
#pragma unroll
                for (int a = 1; a < K; ++a)
                    ldst[a - 1] = T[a];
                if (u + 2 <= kWavePF) {
#pragma unroll
                    for (int ch = 0; ch < C; ++ch)
                        yb[u & 1][ch] = *reinterpret_cast<const float *>(ring_at(t + 2) + ch * kPlane);
                }
                int e = t + 64;
                e = e < wb.log_steps ? e : wb.log_steps - 1;     // past the upper band's last step: unused
#pragma unroll
                for (int a = 1; a < K; ++a)
                    Mn[a] = log_in[e * (K - 1) + a - 1];
            }
            __builtin_amdgcn_sched_barrier(0);
            // ---- the matrix instructions: messages for the rows below, T[a] = S[a+1] + this row's taps
#pragma unroll
            for (int i = 0; i < C; ++i)
                xh[i][0] = xn[i];
#pragma unroll
            for (int a = 1; a < K; ++a) {
                f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
                if (a + 1 < K) {
#pragma unroll
                    for (int o = 0; o < C; ++o)
                        acc[o] = from_lane_above_or(M[a + 1][o], T[a + 1][o]);
                }
#pragma unroll
                for (int db = K - 1; db >= 0; --db)     // oldest column first: only db = 0 waits for this step's result
#pragma unroll
                    for (int i = 0; i < C; ++i)
                        acc = __builtin_amdgcn_mfma_f32_4x4x1f32(wA[a][db][i], xh[i][db], acc, 0, 0, 0);
                T[a] = acc;
            }
#pragma unroll
            for (int i = 0; i < C; ++i)
#pragma unroll
                for (int db = K - 1; db >= 1; --db)
                    xh[i][db] = xh[i][db - 1];
            {
                const bool in_row = (unsigned)(t + 1 - r) < (unsigned)W;
                f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int jj = 0; jj < C; ++jj)
                    acc = __builtin_amdgcn_mfma_f32_4x4x1f32(wLi[jj], in_row ? yb[(u + 1) & 1][jj] : 0.0f, acc, 0, 0, 0);
#pragma unroll
                for (int db = K - 1; db >= 1; --db)
#pragma unroll
                    for (int i = 0; i < C; ++i)
                        acc = __builtin_amdgcn_mfma_f32_4x4x1f32(wA[0][db][i], xh[i][db], acc, 0, 0, 0);
                own = acc;
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // the block's results are in the ring (the batch of its last step was issued a whole step ago)
        __hip_atomic_store(wb.io_done, j + 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    // the messages of the last step, then the whole log is published
    if (r == 63) {
        const int tl = nblocks * kWavePF;
        f32x4 *ldst = log_out + (tl - 1) * (K - 1);
#pragma unroll
        for (int a = 1; a < K; ++a)
            ldst[a - 1] = T[a];
    }
    __hip_atomic_store(wb.prog_out, nblocks * kWavePF, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
}

}  // namespace invconv
