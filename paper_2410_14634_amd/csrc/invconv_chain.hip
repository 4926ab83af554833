// Chain of band-systolic solves in ONE launch: a stack of inverse-convolution
// layers (Section 4.1 stacks K flow steps) solved as a pipeline over layers.
// gfx950 only.
//
// The solve of layer s+1 at pixel p needs the output of layer s only at pixels
// <= p (same partial order as inside a layer, Section 3), so layer s+1 can trail
// layer s by a few dozen anti-diagonals instead of waiting for it to finish.  One
// workgroup per (stage s, image n); workgroups of later stages have higher block
// indices than the ones they wait for.  The same holds for the backward chain in
// mirrored coordinates (the transposed solve of layer l consumes dL/dy of layer
// l+1), so "stage" is simply the processing order the host passes in.
//
// Inside a workgroup
//   waves 0..NB-1   compute: the band-systolic solve on 16x16x4 MFMA of the
//                   single-layer kernel, one wave per 16-row band, but all
//                   operands come from / go to an LDS ring, never global memory;
//   4 loader waves  fetch the input into the ring, after waiting for the producer
//                   stage's progress counter;
//   4 storer waves  drain finished results from the ring to global memory, then
//                   publish the stage's progress.
// Global memory is touched 64 bytes of a row at a time: a group of 16 steps of a
// band is 16 rows x 16 columns per channel, lane (row, quarter) moves 16 bytes,
// the four lanes of a row 64 contiguous bytes.  A group lives in the registers of
// its loader (storer) wave and passes to (from) the ring a quarter, 4 steps, at a
// time, every fourth step.  Each such wave serves two bands whose groups are 6
// and 10 steps out of phase: what it fetched is first used four steps later, a
// storer publishes a group two steps after storing it, and the wave's other
// memory operations are at least four steps old by then, so "wait for everything
// outstanding" costs nothing extra and a memory round trip has four steps to
// finish instead of lying on every step's path.  Every role runs a loop of its
// own (same number of barriers), so its registers are its own.
// Data that crosses workgroups is written and read with agent-scope (device-
// coherent) stores and loads, so publishing needs no cache write-back or
// invalidate: the storer waits until all its stores are acknowledged and then
// advances the counter; the loader reads the counter and only then issues loads.
// The ring is indexed by the global step t (16 slots per row) and is skew-free:
// at step t every row of a band touches slot t, whatever its column, so its
// length covers only the load lead and the store lag, not the 16-column skew of
// a band.  A slot first holds the input y of its step and is then overwritten
// in place by the result x.  All waves meet at one workgroup barrier per step.
#include "invconv_common.h"
#include "invconv_launch.h"

namespace invconv {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// 16 bytes at any 4-byte boundary of one image (a raw buffer of `bytes` bytes), read or written
// device-coherently (sc1): no cache of this or another XCD answers with a stale line.  `lane_off`
// is the lane's byte offset, `plane_off` a wave-uniform one.
constexpr int kCoherent = 16;     // cache policy bit of the buffer instructions that sets sc1
__device__ __forceinline__ __amdgpu_buffer_rsrc_t chain_image_buffer(const float *p, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(p), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ f32x4 chain_load16(__amdgpu_buffer_rsrc_t r, unsigned lane_off, unsigned plane_off)
{
    return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)lane_off, (int)plane_off, kCoherent));
}
__device__ __forceinline__ void chain_store16(__amdgpu_buffer_rsrc_t r, unsigned lane_off, unsigned plane_off, f32x4 v)
{
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), r, (int)lane_off, (int)plane_off, kCoherent);
}

__device__ __forceinline__ float chain_from_row_above(float v)
{
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x111 /* row_shr:1 */, 0xf, 0xf, true));
}

constexpr int kCRing = 16;        // ring slots (steps) per band
constexpr int kCRow = 18;         // floats per (channel, row) of the ring: 16 slots + 2, so that the 16 rows of a
                                  // band fall into 16 different banks and a quarter (4 slots) is two 8-byte words
constexpr int kCBlk = 4;          // steps per ring transfer (a quarter of a group)
constexpr int kCGroup = 16;       // steps per global-memory transfer: 16 columns = 64 bytes of a row
constexpr int kCMsg = 4;          // depth of the band-to-band message ring
constexpr int kCDelay = 1;        // extra steps a band lags behind the band above
constexpr int kCAhead = 2;        // a quarter enters the ring this many steps before its first step is solved
constexpr int kCLead = kCAhead + 4;  // a group is fetched this many steps before its first step: four for the round trip
constexpr int kCPubLag = 2;       // a storer publishes a group this many steps after storing it
constexpr int kCIo = 4;           // loader waves = storer waves
constexpr int kCFlags = 8;        // progress counters per (stage, image): one per band
constexpr int kCSpinLimit = 1 << 21;   // polls (512 clocks apart) of a producer's counter before a loader gives up
constexpr int kCDone = 1 << 30;   // progress value published when a stage has finished

// 16 channels: a loader or storer wave has registers for one band only, so at most 4 bands (64 rows)
__host__ __device__ constexpr int chain_io_bands(int C) { return C <= 12 ? 2 : 1; }

// MAP: a stage may carry a per-pixel affine channel map of a flow step (a.map[stage] != null; C*C floats A,
// then C floats d, true channel order).  In the plain orientation it is applied to the RESULT on its way
// to memory: the compute wave forms A x + d with CG more matrix instructions (the same shape as Linv y: the
// lane's own value in, the lane's own channels out) and puts that into the ring slot instead of x - the
// recurrence keeps x in registers, the ring is only the way out.  In the mirrored orientation its transpose
// is applied to the INPUT, g = A^T (input): the input enters the solve only through Linv y, so the map is
// folded into Linv once and costs nothing per step.
template <int CG, int K, int DIR, bool MAP = false>
__global__ __launch_bounds__(64 * (kCIo * chain_io_bands(4 * CG) + 2 * kCIo)) void k_chain_band(ChainArgs a)
{
    constexpr int C = 4 * CG;
    constexpr int kCIoBands = chain_io_bands(C);     // bands per loader / storer wave
    // Mirrored direction: the four slots of a quarter hold their steps in descending order, which is the
    // ascending memory order, so that loaders and storers move a lane's 16 bytes without reordering them.
    constexpr int kSlotFlip = DIR ? 3 : 0;
    extern __shared__ float smem[];
    const int H = a.H, W = a.W, NB = a.NB;
    const int stage = blockIdx.x / a.B, n_img = blockIdx.x % a.B;
    const float *in = stage == 0 ? a.in0 : a.out[stage - 1];
    float *out = a.out[stage];
    const float *w = a.w[stage];

    float *sLinv = smem;
    float *sCf = sLinv + C * C;
    float *sMsg = sCf + K * K * C * C;               // [NB][kCMsg][K][64]
    float *ring = sMsg + NB * kCMsg * K * 64;        // [NB][C][16 rows][kCRow]; step t of band b is slot (t - b) & 15 of its row
    float *sL = ring;                                // folding scratch, dead before the ring is used
    float *sW = ring + C * C;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    fold_weights_staged<DIR, C>(w, C, K, sL, sLinv, sCf, sW);
    const float *__restrict__ map = MAP ? a.map[stage] : nullptr;
    if (MAP && DIR && map) {
        // solve channel m is true channel C-1-m: the solve's input is y'[m] = sum_j A[C-1-j][C-1-m] in[j],
        // so Linv <- Linv T with T[m][j] = A[C-1-j][C-1-m]  (scratch: the folding buffers, dead by now)
        for (int idx = tid; idx < C * C; idx += blockDim.x) {
            const int o = idx / C, j = idx % C;
            float acc = 0.0f;
            for (int m = 0; m < C; ++m)
                acc += sLinv[o * C + m] * map[(C - 1 - j) * C + (C - 1 - m)];
            sL[idx] = acc;
        }
        __syncthreads();
        for (int idx = tid; idx < C * C; idx += blockDim.x)
            sLinv[idx] = sL[idx];
        __syncthreads();
    }

    const int nrow = lane & 15, g = lane >> 4;       // compute: row of the band, channel group; i/o: row, quarter
    const int span = 16 + W - 1;                               // active steps of a band
    const int t_last = (NB - 1) * (16 + kCDelay) + span;       // one past the last active step of any band
    const int t_end = t_last + kCGroup;                        // a band's last group is stored up to 16 steps later
    const int t_begin = -(kCLead + kCGroup);                   // the group that holds step 0 is fetched up to 22 steps before
    const size_t img = (size_t)n_img * C * H * W;

    if (wave < NB) {
        // ================= compute =================
        const int band = wave;
        float wA[K][K][CG], wLi[CG];
        {
            const int m = nrow;
            const bool m_ok = (m & 3) < CG;
            const int om = m_ok ? CG * (m >> 2) + (m & 3) : 0;
#pragma unroll
            for (int aa = 0; aa < K; ++aa)
#pragma unroll
                for (int db = 0; db < K; ++db)
#pragma unroll
                    for (int jj = 0; jj < CG; ++jj) {
                        const float cf = sCf[((aa * K + db) * C + om) * C + CG * g + jj];
                        wA[aa][db][jj] = m_ok ? -cf : 0.0f;
                    }
#pragma unroll
            for (int jj = 0; jj < CG; ++jj) {
                const float lv = sLinv[om * C + CG * g + jj];
                wLi[jj] = m_ok ? lv : 0.0f;
            }
        }
        // output map of a flow step (plain orientation): weights laid out like wLi, bias per own channel
        float wAz[CG], dz[CG];
        const bool mapped = MAP && !DIR && map != nullptr;
        if (MAP && !DIR) {
            const int m = nrow;
            const bool m_ok = (m & 3) < CG;
            const int om = m_ok ? CG * (m >> 2) + (m & 3) : 0;
#pragma unroll
            for (int jj = 0; jj < CG; ++jj) {
                const float av = mapped ? map[om * C + CG * g + jj] : 0.0f;
                wAz[jj] = m_ok ? av : 0.0f;
                dz[jj] = mapped ? map[C * C + CG * g + jj] : 0.0f;
            }
        }
        __syncthreads();        // everyone is done with sCf/sLinv reads and the folding scratch
        for (int idx = tid; idx < NB * kCMsg * K * 64 + NB * C * 16 * kCRow; idx += blockDim.x)
            sMsg[idx] = 0.0f;   // message ring and data ring are contiguous
        __syncthreads();

        float xh[CG][K];
        f32x4 T[K];
        f32x4 own = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int jj = 0; jj < CG; ++jj)
#pragma unroll
            for (int db = 0; db < K; ++db)
                xh[jj][db] = 0.0f;
#pragma unroll
        for (int aa = 0; aa < K; ++aa)
            T[aa] = f32x4{0.f, 0.f, 0.f, 0.f};
        const int tf_c = band * (16 + kCDelay);                    // first step of this band
        const bool first_row = (nrow == 0) && (band > 0);
        const bool last_row = (nrow == 15) && (band + 1 < NB);
        const float *msg_in = sMsg + (size_t)(band > 0 ? band - 1 : 0) * kCMsg * K * 64 + g * 4;
        float *msg_out = sMsg + (size_t)band * kCMsg * K * 64 + g * 4;
        // ring address of this lane for channel jj at step t: cbase[jj] + ((t - band) & 15)
        int cbase[CG];
#pragma unroll
        for (int jj = 0; jj < CG; ++jj)
            cbase[jj] = ((band * C + CG * g + jj) * 16 + nrow) * kCRow;

        // A step in this order: the terms that need nothing newer than the previous pixel of the row
        // go to the matrix cores first (18 of the 27 products), so that the LDS reads of this step
        // complete behind them; then the pixel itself, then the 9 products that contain it.
        for (int t = t_begin; t < t_end; ++t) {
            const int tau = t - tf_c;
            const int c = tau - nrow;
            // tau = -1 only prepares pixel 0; doing the rest of the step on the all-zero state is harmless
            if (tau >= -1 && tau < span) {
                float yv[CG];
#pragma unroll
                for (int jj = 0; jj < CG; ++jj)
                    yv[jj] = ring[cbase[jj] + (((t + 1 - band) & (kCRing - 1)) ^ kSlotFlip)];
                const float *mi = msg_in + ((t - 1 - kCDelay) & (kCMsg - 1)) * K * 64;
                float mrow[K][CG];
#pragma unroll
                for (int aa = 1; aa < K; ++aa)
#pragma unroll
                    for (int j = 0; j < CG; ++j)
                        mrow[aa][j] = mi[aa * 64 + j];
                const bool in_row = (unsigned)(c + 1) < (unsigned)W;
                // xh[.][db] = x at column c - db (db >= 1); xh[.][0] is filled below
                f32x4 accT[K];
#pragma unroll
                for (int aa = K - 1; aa >= 1; --aa) {      // the last one first: it takes nothing from the row above
                    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
                    if (aa + 1 < K) {
#pragma unroll
                        for (int j = 0; j < CG; ++j) {
                            const float up = chain_from_row_above(T[aa + 1][j]);
                            acc[j] = first_row ? mrow[aa + 1][j] : up;
                        }
                    }
#pragma unroll
                    for (int db = K - 1; db >= 1; --db)
#pragma unroll
                        for (int jj = 0; jj < CG; ++jj)
                            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(wA[aa][db][jj], xh[jj][db], acc, 0, 0, 0);
                    accT[aa] = acc;
                }
                // the part of the next pixel that does not depend on this one
                f32x4 accO = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int db = K - 1; db >= 2; --db)
#pragma unroll
                    for (int jj = 0; jj < CG; ++jj)
                        accO = __builtin_amdgcn_mfma_f32_16x16x4f32(wA[0][db][jj], xh[jj][db - 1], accO, 0, 0, 0);
#pragma unroll
                for (int jj = 0; jj < CG; ++jj)
                    accO = __builtin_amdgcn_mfma_f32_16x16x4f32(wLi[jj], in_row ? yv[jj] : 0.0f, accO, 0, 0, 0);
                // this pixel
                float xn[CG];
#pragma unroll
                for (int j = 0; j < CG; ++j) {
                    const float up = chain_from_row_above(T[1][j]);
                    xn[j] = own[j] + (first_row ? mrow[1][j] : up);
                }
                // result replaces the input in the ring slot of this step (the storers skip invalid pixels);
                // with an output map that is A x + d, formed behind the products the next step waits for
                if (!(MAP && !DIR && mapped)) {
#pragma unroll
                    for (int j = 0; j < CG; ++j)
                        ring[cbase[j] + (((t - band) & (kCRing - 1)) ^ kSlotFlip)] = xn[j];
                }
#pragma unroll
                for (int aa = 1; aa < K; ++aa) {
                    f32x4 acc = accT[aa];
#pragma unroll
                    for (int jj = 0; jj < CG; ++jj)
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(wA[aa][0][jj], xn[jj], acc, 0, 0, 0);
                    T[aa] = acc;
                }
#pragma unroll
                for (int jj = 0; jj < CG; ++jj)
                    accO = __builtin_amdgcn_mfma_f32_16x16x4f32(wA[0][1][jj], xn[jj], accO, 0, 0, 0);
                own = accO;
                if (MAP && !DIR && mapped) {
                    f32x4 accZ = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int j = 0; j < CG; ++j)
                        accZ[j] = dz[j];
#pragma unroll
                    for (int jj = 0; jj < CG; ++jj)
                        accZ = __builtin_amdgcn_mfma_f32_16x16x4f32(wAz[jj], xn[jj], accZ, 0, 0, 0);
#pragma unroll
                    for (int j = 0; j < CG; ++j)
                        ring[cbase[j] + (((t - band) & (kCRing - 1)) ^ kSlotFlip)] = accZ[j];
                }
                if (last_row) {
                    float *mo = msg_out + (t & (kCMsg - 1)) * K * 64;
#pragma unroll
                    for (int aa = 1; aa < K; ++aa)
#pragma unroll
                        for (int j = 0; j < CG; ++j)
                            mo[aa * 64 + j] = T[aa][j];
                }
#pragma unroll
                for (int jj = 0; jj < CG; ++jj) {
#pragma unroll
                    for (int db = K - 1; db >= 2; --db)
                        xh[jj][db] = xh[jj][db - 1];
                    xh[jj][1] = xn[jj];
                }
            }
            __syncthreads();
        }
        return;
    }

    // ================= loaders and storers =================
    __syncthreads();
    for (int idx = tid; idx < NB * kCMsg * K * 64 + NB * C * 16 * kCRow; idx += blockDim.x)
        sMsg[idx] = 0.0f;
    __syncthreads();
    const int io = wave - NB;                        // 0..3 loaders; 4..7 storers
    const int jq = lane >> 4;                        // lane = (row nrow, quarter jq of a 16-step group)
    // A lane moves 16 bytes: columns c0 .. c0+3 of its row, c0 = U + 4*jq - tf - nrow for the group
    // that starts at step U.  The four lanes of a row cover 64 contiguous bytes.
    // Wave q of either kind serves band A in 0..3 and band A' = 4 + ((A + 2) & 3); groups of band A
    // start at steps = A (mod 16), those of A' at steps = A + 10 (mod 16); a band is served at the
    // steps congruent to it modulo 4.  Loader q has A = q, storer q has A = q - 1 (another SIMD).
    const int q = io & (kCIo - 1);
    const int bandA = io < kCIo ? q : ((q + 3) & 3);
    const int rowW = W;
    const unsigned plane_bytes = 4u * (unsigned)(H * W);
    const __amdgpu_buffer_rsrc_t rin = chain_image_buffer(in + img, plane_bytes * C);
    const __amdgpu_buffer_rsrc_t rout = chain_image_buffer(out + img, plane_bytes * C);
    int bnd[kCIoBands], gph[kCIoBands], tfb[kCIoBands];
#pragma unroll
    for (int bi = 0; bi < kCIoBands; ++bi) {
        bnd[bi] = bi == 0 ? bandA : 4 + ((bandA + 2) & 3);
        gph[bi] = bi == 0 ? bandA : bandA + 10;
        tfb[bi] = bnd[bi] * (16 + kCDelay);
    }

    if (io < kCIo) {
        f32x4 lr[kCIoBands][C];
        bool have[kCIoBands], edge[kCIoBands];
        int dsh[kCIoBands];
#pragma unroll
        for (int bi = 0; bi < kCIoBands; ++bi) {
            have[bi] = false;
            edge[bi] = false;
            dsh[bi] = 0;
#pragma unroll
            for (int ch = 0; ch < C; ++ch)
                lr[bi][ch] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        int seen[kCIoBands];                             // producer progress known so far
        const int *pflag[kCIoBands];
        bool lost = false;                               // a wait ran out: what is fetched from now on counts as NaN
#pragma unroll
        for (int bi = 0; bi < kCIoBands; ++bi) {
            seen[bi] = (stage == 0 || a.flags == nullptr) ? kCDone : 0;
            pflag[bi] = (stage > 0 && a.flags) ? a.flags + ((size_t)(stage - 1) * a.B + n_img) * kCFlags + bnd[bi]
                                                : nullptr;
        }
        for (int t = t_begin; t < t_end; ++t) {
#pragma unroll
            for (int bi = 0; bi < kCIoBands; ++bi) {
                if (((t + kCAhead - gph[bi]) & 3) == 0) {
                    const int b = bnd[bi], tf = tfb[bi];
                    const int uw = t + kCAhead;                     // first step of the quarter written now
                    const int i = ((uw - gph[bi]) >> 2) & 3;        // its position in the group held in registers
                    if (have[bi] && jq == i) {
                        float *dst = ring + ((b * C) * 16 + nrow) * kCRow + ((uw - b) & (kCRing - 1));
                        // lr holds memory order, which is also the slot order of the quarter
                        if (!edge[bi]) {
#pragma unroll
                            for (int ch = 0; ch < C; ++ch) {
                                const float qn = __builtin_nanf("");
                                // (selected here, where the value is used: a select right behind the load
                                // would make the wave wait for it at once)
                                const f32x4 v = lost ? f32x4{qn, qn, qn, qn} : lr[bi][ch];
                                float2 *d2 = reinterpret_cast<float2 *>(dst + ch * 16 * kCRow);
                                d2[0] = float2{v[0], v[1]};
                                d2[1] = float2{v[2], v[3]};
                            }
                        } else {
                            // a group that reaches over an end of the row: the lane's four columns were
                            // fetched from the nearest position inside the row, dsh columns away, so
                            // component m belongs dsh slots further (mirrored) or back, if that is in the quarter
                            const int sh = DIR ? dsh[bi] : -dsh[bi];
                            float *de = dst + sh;
#pragma unroll
                            for (int m = 0; m < 4; ++m) {
                                if ((unsigned)(m + sh) < 4u) {
#pragma unroll
                                    for (int ch = 0; ch < C; ++ch)
                                        de[ch * 16 * kCRow + m] = lost ? __builtin_nanf("") : lr[bi][ch][m];
                                }
                            }
                        }
                    }
                    if (i == 3) {
                        const int U = t + kCLead;                   // the next group: its first quarter is written in 4 steps
                        // Nothing fetched is still unused here except the other band's group, issued six or
                        // more steps ago; waiting now keeps the compiler from waiting between the loads below
                        // for registers it reuses.
                        __builtin_amdgcn_s_waitcnt(0);
                        have[bi] = b < NB && U + kCGroup > tf && U < tf + span;
                        if (have[bi]) {
                            if (seen[bi] < U + kCGroup) {
                                // wait until the producer stage has stored every step of this band below U + 16
                                int spins = 0, v = 0;
                                do {
                                    v = __hip_atomic_load(pflag[bi], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                                    if (v >= U + kCGroup)
                                        break;
                                    __builtin_amdgcn_s_sleep(8);
                                } while (++spins < a.spin_limit);
                                if (v < U + kCGroup) {
                                    // bounded wait ran out: carry on without waiting again (every wave still
                                    // finishes), feed NaN to the solve and tell the caller
                                    if (a.err && lane == 0)
                                        __hip_atomic_store(a.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                                    lost = true;
                                    v = kCDone;
                                }
                                seen[bi] = v;
                                asm volatile("" ::: "memory");   // the loads below are issued after the counter was read
                            }
                            int row = b * 16 + nrow;
                            row = row < H ? row : H - 1;
                            const int c0 = (U + 4 * jq - tf) - nrow;
                            const int cv = c0 < 0 ? 0 : (c0 > rowW - 4 ? rowW - 4 : c0);
                            dsh[bi] = c0 - cv;
                            edge[bi] = __builtin_amdgcn_ballot_w64(c0 != cv) != 0;
                            const unsigned off =
                                4u * (unsigned)(DIR ? (H - 1 - row) * rowW + (rowW - 4 - cv) : row * rowW + cv);
#pragma unroll
                            for (int ch = 0; ch < C; ++ch) {
                                // device-coherent: another workgroup of this launch may have written it
                                lr[bi][ch] = chain_load16(rin, off, plane_bytes * (unsigned)(DIR ? C - 1 - ch : ch));
                            }
                        }
                    }
                }
            }
            __syncthreads();
        }
        return;
    }

    // ---- storer
    int *myflag[kCIoBands];
    f32x4 sr[kCIoBands][C];
    int publish[kCIoBands], pubat[kCIoBands];        // progress to publish once the band's stores are acknowledged, and when
#pragma unroll
    for (int bi = 0; bi < kCIoBands; ++bi) {
        myflag[bi] = a.flags ? a.flags + ((size_t)stage * a.B + n_img) * kCFlags + bnd[bi] : nullptr;
        publish[bi] = 0;
        pubat[bi] = 0;
#pragma unroll
        for (int ch = 0; ch < C; ++ch)
            sr[bi][ch] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    for (int t = t_begin; t < t_end; ++t) {
#pragma unroll
        for (int bi = 0; bi < kCIoBands; ++bi) {
            // The band's last stores were issued kCPubLag steps ago (the other band's four or more), as
            // device-coherent stores; once all are acknowledged, every step below `publish` is in memory.
            if (myflag[bi] && publish[bi] > 0 && t >= pubat[bi]) {
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_waitcnt(0);
                asm volatile("" ::: "memory");
                if (lane == 0)
                    __hip_atomic_store(myflag[bi], publish[bi], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                publish[bi] = 0;
            }
            if (((t - gph[bi]) & 3) == 0) {
                const int b = bnd[bi], tf = tfb[bi];
                // collect the quarter [t-4, t); after the fourth quarter store the group
                const int us = t - kCBlk;
                const int i = ((us - gph[bi]) >> 2) & 3;
                if (b < NB && us + kCBlk > tf && us < tf + span && jq == i) {
                    const float *src = ring + ((b * C) * 16 + nrow) * kCRow + ((us - b) & (kCRing - 1));
#pragma unroll
                    for (int ch = 0; ch < C; ++ch) {
                        // memory order (mirrored: columns descending) = slot order: the store needs no shuffle
                        const float2 *s2 = reinterpret_cast<const float2 *>(src + ch * 16 * kCRow);
                        const float2 lo = s2[0], hi = s2[1];
                        sr[bi][ch] = f32x4{lo.x, lo.y, hi.x, hi.y};
                    }
                }
                if (i == 3) {
                    const int U = us - 3 * kCBlk;
                    if (b < NB && U + kCGroup > tf && U < tf + span) {
                        const int row = b * 16 + nrow;
                        const int c0 = (U + 4 * jq - tf) - nrow;
                        if (row < H && c0 >= 0 && c0 + 3 <= rowW - 1) {
                            const unsigned off =
                                4u * (unsigned)(DIR ? (H - 1 - row) * rowW + (rowW - 4 - c0) : row * rowW + c0);
#pragma unroll
                            for (int ch = 0; ch < C; ++ch)
                                chain_store16(rout, off, plane_bytes * (unsigned)(DIR ? C - 1 - ch : ch), sr[bi][ch]);
                        } else if (row < H) {
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                const int cj = c0 + j;
                                if ((unsigned)cj < (unsigned)rowW) {
                                    const unsigned offj = 4u * (unsigned)(DIR ? (H - 1 - row) * rowW + (rowW - 1 - cj)
                                                                              : row * rowW + cj);
#pragma unroll
                                    for (int ch = 0; ch < C; ++ch) {
                                        char *base = reinterpret_cast<char *>(
                                            out + img + (size_t)(DIR ? C - 1 - ch : ch) * H * rowW);
                                        __hip_atomic_store(reinterpret_cast<float *>(base + offj),
                                                           sr[bi][ch][DIR ? 3 - j : j], __ATOMIC_RELAXED,
                                                           __HIP_MEMORY_SCOPE_AGENT);
                                    }
                                }
                            }
                        }
                    }
                    publish[bi] = t;                    // = U + 16: everything below it has now been issued
                    pubat[bi] = t + kCPubLag;
                }
            }
        }
        __syncthreads();
    }
    // everything is drained: tell the consumer stage it never has to wait again
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0);
    asm volatile("" ::: "memory");
#pragma unroll
    for (int bi = 0; bi < kCIoBands; ++bi)
        if (myflag[bi] && lane == 0)
            __hip_atomic_store(myflag[bi], kCDone, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ void k_chain_clear(int *flags, int nflags)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nflags)
        flags[i] = 0;
}

size_t chain_lds_bytes(int C, int k, int NB)
{
    return sizeof(float) * ((size_t)C * C + (size_t)k * k * C * C + (size_t)NB * kCMsg * k * 64 +
                            (size_t)NB * C * 16 * kCRow);
}

bool chain_supported(int stages, int C, int H, int W, int k)
{
    // W >= 4: a lane moves four columns of a row at a time
    return stages >= 1 && stages <= kChainMaxLayers && (C == 8 || C == 12 || C == 16) && k == 3 && W >= 4 &&
           (H + 15) / 16 <= kCIo * chain_io_bands(C) &&
           chain_lds_bytes(C, k, (H + 15) / 16) <= kMaxLdsBytes;
}

// One layer: the band kernel (one wave per band, every lane walking its own row four bytes at a time)
// keeps B*H*C*2 cache lines of 128 bytes live; beyond about 2 MB per XCD (an eighth of them on each)
// its lines are evicted between two touches and it collapses (B = 256, 12 x 128 x 128: 1.3 ms against
// 0.3 ms), while this kernel moves whole 64-byte pieces and does not care.  Below that the band kernel
// wins on small images (this kernel runs 38 steps more), this one on tall ones (measured: 253 against
// 293 us at B = 32, 12 x 128 x 128).
bool chain_single_preferred(int B, int C, int H)
{
    // (images of one band, H <= 16, stay on the band kernel whatever the batch: there this kernel would keep one
    // of its eight solving waves busy - 1024 x 12x16x16: 40 us on the band kernel, 125 us here; 4096: 133 / 492 us)
    // With two bands (H <= 32) it keeps two of eight, and takes over later: 700 x 12x24x24 94 against 146 us,
    // 400 x 12x20x20 56 / 93; 1024 x 12x32x32 385 / 215.
    const double live_per_xcd = (double)B * H * C * 256.0 / 8.0;
    if (H <= 16)
        return false;
    if (H <= 32)      // (16 channels: the band kernel's registers allow fewer waves, it falls behind sooner: 256 x 16x32x32 112 us)
        return live_per_xcd > (C == 16 ? 3.0e6 : 8.0e6);
    return live_per_xcd > 2.0e6 || (H > 80 && B >= 24);
}

size_t chain_flag_ints(int stages, int B) { return (size_t)stages * B * kCFlags; }

// A workgroup of stage s waits for the workgroup of stage s-1 of the same image, so a launch holds at most
// as many workgroups as the device keeps resident at once: then nothing depends on the order in which the
// hardware starts them.  A longer stack goes out as several launches of whole stages (a launch's first
// stage reads what the launch before it has finished, without waiting); a batch that is too large for
// even one launch of two stages goes out stage by stage, where no workgroup waits for another.
template <int CG, int K>
static int launch_chain_ck(int dir, const ChainArgs &all, int C, hipStream_t stream)
{
    bool mapped = false;
    for (int s = 0; s < all.stages; ++s)
        mapped = mapped || all.map[s] != nullptr;
    const size_t lds = chain_lds_bytes(C, K, all.NB);
    const void *fn = mapped ? (dir ? reinterpret_cast<const void *>(&k_chain_band<CG, K, 1, true>)
                                   : reinterpret_cast<const void *>(&k_chain_band<CG, K, 0, true>))
                            : (dir ? reinterpret_cast<const void *>(&k_chain_band<CG, K, 1>)
                                   : reinterpret_cast<const void *>(&k_chain_band<CG, K, 0>));
    if (!ensure_dynamic_lds(fn, lds))
        return INVCONV_ERR_UNSUPPORTED;
    const int threads = 64 * (all.NB + 2 * kCIo);
    int per_launch = all.stages;                    // stages per launch
    if (all.stages > 1) {
        const int resident = resident_workgroups(fn, threads, lds);
        per_launch = resident / all.B;
        if (per_launch < 1)
            per_launch = 1;
        if (per_launch > all.stages)
            per_launch = all.stages;
    }
    for (int s0 = 0; s0 < all.stages; s0 += per_launch) {
        ChainArgs a = all;
        a.stages = all.stages - s0 < per_launch ? all.stages - s0 : per_launch;
        a.in0 = s0 == 0 ? all.in0 : all.out[s0 - 1];
        for (int s = 0; s < a.stages; ++s) {
            a.w[s] = all.w[s0 + s];
            a.out[s] = all.out[s0 + s];
            a.map[s] = all.map[s0 + s];
        }
        if (a.stages > 1) {
            const int nflags = a.stages * a.B * kCFlags;
            hipLaunchKernelGGL(k_chain_clear, dim3((nflags + 255) / 256), dim3(256), 0, stream, a.flags, nflags);
            if (hipGetLastError() != hipSuccess)
                return INVCONV_ERR_LAUNCH;
        } else {
            a.flags = nullptr;      // one stage: nothing to wait for, nothing to publish
        }
        const dim3 grid((unsigned)(a.stages * a.B)), block((unsigned)threads);
        if (mapped && dir)
            hipLaunchKernelGGL((k_chain_band<CG, K, 1, true>), grid, block, lds, stream, a);
        else if (mapped)
            hipLaunchKernelGGL((k_chain_band<CG, K, 0, true>), grid, block, lds, stream, a);
        else if (dir)
            hipLaunchKernelGGL((k_chain_band<CG, K, 1>), grid, block, lds, stream, a);
        else
            hipLaunchKernelGGL((k_chain_band<CG, K, 0>), grid, block, lds, stream, a);
        if (hipGetLastError() != hipSuccess)
            return INVCONV_ERR_LAUNCH;
    }
    return INVCONV_OK;
}

// Runs `stages` solves as pipelined launches.  args.flags (chain_flag_ints() ints) may be null only when
// stages == 1; args.err is the caller's error word or null.
int launch_chain(int dir, ChainArgs args, int C, int k, hipStream_t stream)
{
    if (!chain_supported(args.stages, C, args.H, args.W, k) || (args.stages > 1 && !args.flags))
        return INVCONV_ERR_VARIANT;
    args.NB = (args.H + 15) / 16;
    args.spin_limit = wait_budget(kCSpinLimit);
    if (C == 8) return launch_chain_ck<2, 3>(dir, args, C, stream);
    if (C == 12) return launch_chain_ck<3, 3>(dir, args, C, stream);
    if (C == 16) return launch_chain_ck<4, 3>(dir, args, C, stream);
    return INVCONV_ERR_VARIANT;
}

}  // namespace invconv
