// Chain of band-systolic solves in ONE launch: a stack of inverse-convolution
// layers (Section 4.1 stacks K flow steps) solved as a pipeline over layers.
// gfx950 only.
//
// The solve of layer s+1 at pixel p needs the output of layer s only at pixels
// <= p (same partial order as inside a layer, Section 3), so layer s+1 can trail
// layer s by a few anti-diagonals instead of waiting for it to finish.  One
// workgroup per (stage s, image n); workgroups of later stages have higher block
// indices than the ones they wait for.  The same holds for the backward chain in
// mirrored coordinates (the transposed solve of layer l consumes dL/dy of layer
// l+1), so "stage" is simply the processing order the host passes in.
//
// Inside a workgroup
//   waves 0..NB-1   compute: the band-systolic solve on 16x16x4 MFMA of the
//                   single-layer kernel, one wave per 16-row band, but all
//                   operands come from / go to an LDS ring, never global memory;
//   4 loader waves  fetch the input in blocks of 4 steps (16 rows x 4 columns
//                   per instruction, so a row contributes 16 contiguous bytes)
//                   into the ring, after waiting for the producer stage's
//                   progress counter;
//   4 storer waves  drain finished results from the ring to global memory in
//                   the same blocks, then publish the stage's progress.
// Loader and storer wave q serve bands q and q+4, and only at steps congruent
// to q modulo 4: what a loader fetched is written into the ring four steps
// later, and a storer publishes a block four steps after storing it.  The wave
// issues no other memory operation in between, so "wait for everything
// outstanding" is exact and a memory round trip has four steps to finish instead
// of lying on every step's path.  Every role runs a loop of its own (same number
// of barriers), so its registers are its own.
// Data that crosses workgroups is written and read with agent-scope (device-
// coherent) stores and loads, so publishing needs no cache write-back or
// invalidate: the storer waits until all its stores are acknowledged and then
// advances the counter; the loader reads the counter and only then issues loads.
// The ring is indexed by the global step t (slot t mod 16) and is skew-free:
// at step t every row of a band touches slot t, whatever its column, so its
// length covers only the load lead and the store lag, not the 16-column skew of
// a band.  A slot first holds the input y of its step and is then overwritten
// in place by the result x.  All waves meet at one workgroup barrier per step.
#include "invconv_common.h"
#include "invconv_launch.h"

namespace invconv {

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float chain_from_row_above(float v)
{
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x111 /* row_shr:1 */, 0xf, 0xf, true));
}

constexpr int kCRing = 16;        // ring slots (steps) per band
constexpr int kCBlk = 4;          // steps per load/store block
constexpr int kCMsg = 4;          // depth of the band-to-band message ring
constexpr int kCDelay = 1;        // extra steps a band lags behind the band above
constexpr int kCLead = 8;         // a block is loaded this many steps before its first step
constexpr int kCIo = 4;           // loader waves = storer waves = flags per (stage, image)
constexpr int kCIoBands = 2;      // bands per loader / storer wave (NB <= 8)
constexpr int kCSpinLimit = 1 << 21;
constexpr int kCDone = 1 << 30;   // progress value published when a stage has finished

template <int CG, int K, int DIR>
__global__ __launch_bounds__(1024) void k_chain_band(ChainArgs a)
{
    constexpr int C = 4 * CG;
    extern __shared__ float smem[];
    const int H = a.H, W = a.W, NB = a.NB;
    const int stage = blockIdx.x / a.B, n_img = blockIdx.x % a.B;
    const float *in = stage == 0 ? a.in0 : a.out[stage - 1];
    float *out = a.out[stage];
    const float *w = a.w[stage];

    float *sLinv = smem;
    float *sCf = sLinv + C * C;
    float *sMsg = sCf + K * K * C * C;               // [NB][kCMsg][K][64]
    float *ring = sMsg + NB * kCMsg * K * 64;        // [NB][C][kCRing][16]
    float *sL = ring;                                // folding scratch, dead before the ring is used
    float *sW = ring + C * C;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    fold_weights<DIR, C>(w, C, K, sL, sLinv, sCf, sW);

    const int nrow = lane & 15, g = lane >> 4;       // compute: row of the band, channel group; i/o: row, step of the block
    const int span = 16 + W - 1;                               // active steps of a band
    const int t_last = (NB - 1) * (16 + kCDelay) + span;       // one past the last active step of any band
    const int t_end = t_last + kCBlk;                          // a band's last steps are drained up to 4 steps later
    const int t_begin = -(kCLead + kCBlk);
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
        __syncthreads();        // everyone is done with sCf/sLinv reads and the folding scratch
        for (int idx = tid; idx < NB * kCMsg * K * 64 + NB * C * kCRing * 16; idx += blockDim.x)
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
        // ring address of this lane for channel jj at slot s: cbase[jj] + s*16
        int cbase[CG];
#pragma unroll
        for (int jj = 0; jj < CG; ++jj)
            cbase[jj] = ((band * C + CG * g + jj) * kCRing) * 16 + nrow;

        for (int t = t_begin; t < t_end; ++t) {
            const int tau = t - tf_c;
            const int c = tau - nrow;
            if (tau >= 0 && tau < span) {
                const float *mi = msg_in + ((t - 1 - kCDelay) & (kCMsg - 1)) * K * 64;
                float mrow[K][CG];
#pragma unroll
                for (int aa = 1; aa < K; ++aa)
#pragma unroll
                    for (int j = 0; j < CG; ++j)
                        mrow[aa][j] = mi[aa * 64 + j];
                float xn[CG];
#pragma unroll
                for (int j = 0; j < CG; ++j) {
                    const float up = chain_from_row_above(T[1][j]);
                    xn[j] = own[j] + (first_row ? mrow[1][j] : up);
                }
                // result replaces the input in the ring slot of this step (the storers skip invalid pixels)
#pragma unroll
                for (int j = 0; j < CG; ++j)
                    ring[cbase[j] + (t & (kCRing - 1)) * 16] = xn[j];
#pragma unroll
                for (int jj = 0; jj < CG; ++jj)
                    xh[jj][0] = xn[jj];
#pragma unroll
                for (int aa = 1; aa < K; ++aa) {
                    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
                    if (aa + 1 < K) {
#pragma unroll
                        for (int j = 0; j < CG; ++j) {
                            const float up = chain_from_row_above(T[aa + 1][j]);
                            acc[j] = first_row ? mrow[aa + 1][j] : up;
                        }
                    }
#pragma unroll
                    for (int db = K - 1; db >= 0; --db)     // oldest column first: only db = 0 waits for this step's result
#pragma unroll
                        for (int jj = 0; jj < CG; ++jj)
                            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(wA[aa][db][jj], xh[jj][db], acc, 0, 0, 0);
                    T[aa] = acc;
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
                for (int jj = 0; jj < CG; ++jj)
#pragma unroll
                    for (int db = K - 1; db >= 1; --db)
                        xh[jj][db] = xh[jj][db - 1];
            }
            if (tau + 1 >= 0 && tau + 1 < span) {
                // prepare the part of the next pixel that does not depend on the rows above
                const bool in_row = (unsigned)(c + 1) < (unsigned)W;
                f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int jj = 0; jj < CG; ++jj) {
                    const float yv = ring[cbase[jj] + ((t + 1) & (kCRing - 1)) * 16];
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(wLi[jj], in_row ? yv : 0.0f, acc, 0, 0, 0);
                }
#pragma unroll
                for (int db = K - 1; db >= 1; --db)
#pragma unroll
                    for (int jj = 0; jj < CG; ++jj)
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(wA[0][db][jj], xh[jj][db], acc, 0, 0, 0);
                own = acc;
            }
            __syncthreads();
        }
        return;
    }

    // ================= loaders and storers =================
    __syncthreads();
    for (int idx = tid; idx < NB * kCMsg * K * 64 + NB * C * kCRing * 16; idx += blockDim.x)
        sMsg[idx] = 0.0f;
    __syncthreads();
    const int io = wave - NB;                        // 0..3 loaders; 4..7 storers
    const int q = io & (kCIo - 1);                   // serves bands q, q + 4 at steps = q (mod 4)
    const int jblk = lane >> 4;                      // lane = (row nrow, step jblk of the block)

    if (io < kCIo) {
        float lreg[kCIoBands][C];
        bool have[kCIoBands];
#pragma unroll
        for (int bi = 0; bi < kCIoBands; ++bi) {
            have[bi] = false;
#pragma unroll
            for (int ch = 0; ch < C; ++ch)
                lreg[bi][ch] = 0.0f;
        }
        int seen = (stage == 0 || a.flags == nullptr) ? kCDone : 0;   // producer progress known so far
        const int *pflag =
            (stage > 0 && a.flags) ? a.flags + ((size_t)(stage - 1) * a.B + n_img) * kCIo + q : nullptr;
        const bool coherent = stage > 0;
        for (int t = t_begin; t < t_end; ++t) {
            if ((t & (kCIo - 1)) == q) {
                const int uw = t + kCLead - kCBlk;          // first step of the block to write (fetched 4 steps ago)
                const int ul = t + kCLead;                  // first step of the block to fetch
#pragma unroll
                for (int bi = 0; bi < kCIoBands; ++bi) {
                    const int b = q + kCIo * bi;
                    if (have[bi]) {
                        const int slot = (uw + jblk) & (kCRing - 1);
#pragma unroll
                        for (int ch = 0; ch < C; ++ch)
                            ring[((b * C + ch) * kCRing + slot) * 16 + nrow] = lreg[bi][ch];
                    }
                }
#pragma unroll
                for (int bi = 0; bi < kCIoBands; ++bi) {
                    const int b = q + kCIo * bi;
                    const int tf = b * (16 + kCDelay);
                    have[bi] = b < NB && ul + kCBlk > tf && ul < tf + span;
                    if (have[bi]) {
                        if (seen < ul + kCBlk) {
                            // wait until the producer stage has stored every step below ul + kCBlk
                            int spins = 0, v = 0;
                            do {
                                v = __hip_atomic_load(pflag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                                if (v >= ul + kCBlk)
                                    break;
                                __builtin_amdgcn_s_sleep(8);
                            } while (++spins < kCSpinLimit);
                            if (v < ul + kCBlk) {
                                if (a.err)
                                    a.err[0] = 1;       // bounded wait ran out: carry on, results are invalid
                                v = kCDone;
                            }
                            seen = v;
                            asm volatile("" ::: "memory");   // the loads below are issued after the counter was read
                        }
                        int row = b * 16 + nrow;
                        row = row < H ? row : H - 1;
                        int cc = (ul + jblk - tf) - nrow;
                        cc = cc < 0 ? 0 : (cc > W - 1 ? W - 1 : cc);
                        const unsigned off = 4u * (unsigned)(DIR ? (H - 1 - row) * W + (W - 1 - cc) : row * W + cc);
#pragma unroll
                        for (int ch = 0; ch < C; ++ch) {
                            const char *base = reinterpret_cast<const char *>(
                                in + img + (size_t)(DIR ? C - 1 - ch : ch) * H * W);
                            const float *src = reinterpret_cast<const float *>(base + off);
                            // what another workgroup of this launch wrote is read device-coherently
                            lreg[bi][ch] = coherent ? __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                                    : *src;
                        }
                    }
                }
            }
            __syncthreads();
        }
        return;
    }

    // ---- storer
    int *myflag = a.flags ? a.flags + ((size_t)stage * a.B + n_img) * kCIo + q : nullptr;
    for (int t = t_begin; t < t_end; ++t) {
        if ((t & (kCIo - 1)) == q) {
            // First publish: this wave's last stores were issued four steps ago, as agent-scope
            // (device-coherent) stores; once they are all acknowledged, its bands have drained every
            // step below t - 4.
            if (myflag && t - kCBlk > 0) {
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_waitcnt(0);
                asm volatile("" ::: "memory");
                if (lane == 0)
                    __hip_atomic_store(myflag, t - kCBlk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            // then drain block [t-4, t) of both bands
            const int us = t - kCBlk;
#pragma unroll
            for (int bi = 0; bi < kCIoBands; ++bi) {
                const int b = q + kCIo * bi;
                const int tf = b * (16 + kCDelay);
                if (b < NB && us + kCBlk > tf && us < tf + span) {
                    const int row = b * 16 + nrow;
                    const int cc = (us + jblk - tf) - nrow;
                    const int slot = (us + jblk) & (kCRing - 1);
                    float val[C];
#pragma unroll
                    for (int ch = 0; ch < C; ++ch)
                        val[ch] = ring[((b * C + ch) * kCRing + slot) * 16 + nrow];
                    if (row < H && (unsigned)cc < (unsigned)W) {
                        const unsigned off = 4u * (unsigned)(DIR ? (H - 1 - row) * W + (W - 1 - cc) : row * W + cc);
#pragma unroll
                        for (int ch = 0; ch < C; ++ch) {
                            char *base = reinterpret_cast<char *>(out + img + (size_t)(DIR ? C - 1 - ch : ch) * H * W);
                            float *dst = reinterpret_cast<float *>(base + off);
                            if (myflag)     // another workgroup of this launch will read it
                                __hip_atomic_store(dst, val[ch], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            else
                                *dst = val[ch];
                        }
                    }
                }
            }
        }
        __syncthreads();
    }
    if (myflag) {
        // everything is drained: tell the consumer stage it never has to wait again
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0);
        asm volatile("" ::: "memory");
        if (lane == 0)
            __hip_atomic_store(myflag, kCDone, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

__global__ void k_chain_clear(int *flags, int nflags, int *err)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nflags)
        flags[i] = 0;
    if (i == 0 && err)
        err[0] = 0;
}

size_t chain_lds_bytes(int C, int k, int NB)
{
    return sizeof(float) * ((size_t)C * C + (size_t)k * k * C * C + (size_t)NB * kCMsg * k * 64 +
                            (size_t)NB * C * kCRing * 16);
}

bool chain_supported(int stages, int C, int H, int k)
{
    return stages >= 1 && stages <= kChainMaxLayers && (C == 8 || C == 12 || C == 16) && k == 3 && H <= 128 &&
           chain_lds_bytes(C, k, (H + 15) / 16) <= kMaxLdsBytes;
}

size_t chain_flag_ints(int stages, int B) { return (size_t)stages * B * kCIo + 64; }

template <int CG, int K>
static int launch_chain_ck(int dir, const ChainArgs &args, int C, hipStream_t stream)
{
    const size_t lds = chain_lds_bytes(C, K, args.NB);
    const void *fn = dir ? reinterpret_cast<const void *>(&k_chain_band<CG, K, 1>)
                         : reinterpret_cast<const void *>(&k_chain_band<CG, K, 0>);
    if (lds > 48 * 1024 &&
        hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
        (void)hipGetLastError();
        return INVCONV_ERR_UNSUPPORTED;
    }
    const dim3 grid((unsigned)(args.stages * args.B)), block((unsigned)(64 * (args.NB + 2 * kCIo)));
    if (dir)
        hipLaunchKernelGGL((k_chain_band<CG, K, 1>), grid, block, lds, stream, args);
    else
        hipLaunchKernelGGL((k_chain_band<CG, K, 0>), grid, block, lds, stream, args);
    return hipGetLastError() == hipSuccess ? INVCONV_OK : INVCONV_ERR_LAUNCH;
}

// Runs `stages` solves as one pipelined launch.  args.flags (chain_flag_ints() ints; the last one is the
// error word) is cleared first; it may be null only when stages == 1.
int launch_chain(int dir, ChainArgs args, int C, int k, hipStream_t stream)
{
    if (!chain_supported(args.stages, C, args.H, k) || (args.stages > 1 && !args.flags))
        return INVCONV_ERR_VARIANT;
    args.NB = (args.H + 15) / 16;
    if (args.flags) {
        const int nflags = args.stages * args.B * kCIo;
        args.err = args.flags + nflags;
        hipLaunchKernelGGL(k_chain_clear, dim3((nflags + 255) / 256), dim3(256), 0, stream, args.flags, nflags,
                           args.err);
        if (hipGetLastError() != hipSuccess)
            return INVCONV_ERR_LAUNCH;
    } else {
        args.err = nullptr;
    }
    if (C == 8) return launch_chain_ck<2, 3>(dir, args, C, stream);
    if (C == 12) return launch_chain_ck<3, 3>(dir, args, C, stream);
    if (C == 16) return launch_chain_ck<4, 3>(dir, args, C, stream);
    return INVCONV_ERR_VARIANT;
}

}  // namespace invconv
