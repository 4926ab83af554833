// Host-side launch interface between the C ABI and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

#include "invconv.h"
#include "invconv_probe.h"

namespace invconv {

constexpr int kSolveBlock = 256;
constexpr int kDwBlock = 256;
constexpr size_t kMaxLdsBytes = 160 * 1024;   // LDS per workgroup on gfx950
constexpr size_t kDwLdsBudget = 40 * 1024;
constexpr int kChainMaxLayers = 16;

// Sets the dynamic-LDS limit of kernel `fn` to at least `bytes` on the current device; the runtime is asked
// once per (device, kernel) and size step, not on every launch.  False if the runtime refuses.
bool ensure_dynamic_lds(const void *fn, size_t bytes);
// Workgroups of kernel `fn` (block of `threads`, `lds` bytes of dynamic LDS) that the current device holds
// at the same time; cached.  0 if the runtime cannot tell.
int resident_workgroups(const void *fn, int threads, size_t lds);
// Polls a bounded wait makes before it gives up: `standard` unless invconv_set_wait_budget() has set another.
int wait_budget(int standard);
void set_wait_budget(int polls);   // 0 restores the standard budgets

// Scratch a caller handed in for one solve.  `base` points behind the workspace header (256-byte aligned),
// `err` at the header's error word; all null / 0 when the call has no workspace.
struct SolveWs {
    char *base = nullptr;
    size_t bytes = 0;
    int *err = nullptr;
};
// Bytes of SolveWs the automatic kernel choice can use for this shape (0: none)
size_t solve_ws_bytes(int B, int C, int H, int W, int k);

struct DwPlan {
    int rt;          // rows per chunk (0 = shape unsupported)
    int nchunks;     // row chunks per image
    int cw, ncol;    // generic pass 1: columns per chunk, column chunks per row chunk (cw = W, ncol = 1 unless W is too wide for LDS)
    int groups;      // matrix-core pass 1: workgroups per image, each looping over chunks
    int ipw;         // matrix-core pass 1: images a workgroup takes one after the other (0 or 1: one; more only for images of a single chunk)
    int cb, cbx;     // matrix-core pass 1: 0, or the output / input channels of a block of dL/dw when the result is formed in blocks (more than 16 channels, or more columns C k k than a wave has accumulators)
    int xw, sxc, svc; // matrix-core pass 1: row and channel strides of the x tile, channel stride of the v tile (padded against LDS bank conflicts)
    size_t nparts;   // workgroups of pass 1 = rows of the partial-sum matrix
    size_t lds;      // dynamic LDS bytes of pass 1
    size_t bytes;    // workspace bytes
};

size_t solve_block_lds_bytes(int C, int H, int k);
int launch_solve_block(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W,
                       int k, hipStream_t stream);
int launch_solve_diag(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W,
                      int k, hipStream_t stream);
int launch_solve_diag_wave(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W, int k,
                           hipStream_t stream);
bool wave_supported(int C, int H, int k);
// `logdet` (may be null): one device float that receives log|det dx/dy| of one image on the side
int launch_solve_wave(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W, int k,
                      hipStream_t stream, float *logdet = nullptr);
bool band_supported(int C, int H, int k);
int launch_solve_band(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W, int k,
                      hipStream_t stream, float *logdet = nullptr);
// one flow step's forward pass (y in, z out, the step's log-determinant on the side) on the one-band kernel
bool flow_band_supported(int C, int H, int k);
int launch_flow_fwd_band(const float *y, const float *w, const float *s, const float *b, const float *Q, float *z,
                         int B, int C, int H, int W, int k, hipStream_t stream, float *logdet);
// many channels (17 .. 48), k = 3: 16x16x4 MFMA per tap, history in an LDS ring
bool wide_supported(int C, int H, int k);
// gw: null, or wide_prefold_ws_bytes(C, H, k) > 0 bytes of device scratch (256-byte aligned): the weights are then
// folded once per call by a set-up launch instead of once per workgroup
size_t wide_prefold_ws_bytes(int C, int H, int k);
int launch_solve_wide(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W, int k,
                      hipStream_t stream, float *logdet = nullptr, float *gw = nullptr);
int launch_wide_fold(int dir, const float *w, float *gw, int C, int k, hipStream_t stream);
// many channels (20 .. 48, multiples of 4) with k = 2, 5, 7, 9, 11: the same solve with its folded weights streamed from
// `gw`, wide_stream_ws_bytes(C, k) bytes of device scratch that a set-up launch of the same call fills
bool wide_stream_supported(int C, int H, int k);
size_t wide_stream_ws_bytes(int C, int k);
int launch_solve_wide_stream(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W, int k,
                             hipStream_t stream, float *gw);
bool bwd_wave_supported(int C, int H, int W, int k);
bool bwd_wave_fused_pays(int B, int C, int H, int W, int k);   // false: solve and weight gradient as separate launches
// one flow step's forward pass (y in, z out, log-determinant of the step on the side) on the split solve, no set-up launch
bool flow_split_supported(int B, int C, int H, int W, int k);
int launch_flow_fwd_split(const float *y, const float *w, const float *s, const float *b, const float *Q, float *z,
                          int B, int C, int H, int W, int k, hipStream_t stream, float *logdet);
// the step's backward pass on eight waves per image (z and dL/dz in; dL/dy and one row [C*C*k*k | C*C | C] per image
// out), and the last kernel that turns those rows into the parameter gradients
bool flow_bwd_split_supported(int B, int C, int H, int W, int k);
int launch_flow_bwd_split(const float *z, const float *w, const float *gz, const float *s, const float *b,
                          const float *Q, float *v, float *part, int B, int C, int H, int W, int k, hipStream_t stream);
int launch_flow_finish_rows(const float *rows, int nrows, const float *w, const float *s, const float *b,
                            const float *Q, float *dLdw, float *dLds, float *dLdb, float *dLdQ, float lw, int C, int H,
                            int W, int k, hipStream_t stream);
int launch_solve_wave_split(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W, int k,
                            hipStream_t stream, float *logdet = nullptr);
bool wave_split_preferred(int B, int H, int W, int k);
bool wave_tile_preferred(int B, int C, int H, int W);
bool wave_bands_supported(int C, int H, int W, int k);
int launch_solve_wave_bands(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W, int k,
                            hipStream_t stream, SolveWs ws = SolveWs{});
size_t wave_bands_ws_bytes(int B, int C, int H, int W, int k);
int launch_bwd_wave(const float *x, const float *w, const float *g, float *v, float *part, int B, int C, int H,
                    int W, int k, hipStream_t stream);
// sign: -1 for the inverse convolution's dL/dw (Theorem 2), +1 for the convolution's own
int launch_dw_reduce(const float *part, int nparts, float *dw, int C, int k, hipStream_t stream, float sign = -1.0f);
int launch_solve_persistent(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W,
                            int k, hipStream_t stream);
int launch_probe(int mode, int steps, int blocks, hipStream_t stream);
DwPlan plan_dw(int B, int C, int H, int W, int k);
int launch_dw(const float *x, const float *v, float *dw, float *part, const DwPlan &p, int B, int C, int H,
              int W, int k, hipStream_t stream, float sign = -1.0f);
bool dw_mfma_supported(int C, int k);
DwPlan plan_dw_mfma(int B, int C, int H, int W, int k);
DwPlan plan_dw_mfma_layers(int layers, int B, int C, int H, int W, int k);
int launch_dw_mfma(const float *x, const float *v, float *dw, float *part, const DwPlan &p, int B, int C, int H,
                   int W, int k, hipStream_t stream, float sign = -1.0f, bool masked = true);
int launch_dw_mfma_partial(const float *x, const float *v, float *part, const DwPlan &p, int B, int C, int H, int W,
                           int k, hipStream_t stream);
int launch_dw_mfma_layers(const float *const *x, const float *const *v, float *const *dw, int layers, float *part,
                          const DwPlan &p, int B, int C, int H, int W, int k, hipStream_t stream);
DwPlan plan_dw_any(int B, int C, int H, int W, int k);
struct PtrList { float *p[kChainMaxLayers]; };
struct ConstPtrList { const float *p[kChainMaxLayers]; };
int launch_dw_reduce_layers(const float *part, int nparts, float *const *dw, int layers, int C, int k,
                            hipStream_t stream, float sign = -1.0f);
// Blocks of a result with more than 16 channels reduced by one launch: block l holds cv[l] x cx[l] k k entries per row
// (rows pstride floats apart, block l's rows start at part + l * nparts * pstride) that go to output channels
// o0[l] .. and input channels i0[l] .. of the Ctot-channel result.
struct DwBlocks {
    int n;
    unsigned char cv[kChainMaxLayers], cx[kChainMaxLayers], o0[kChainMaxLayers], i0[kChainMaxLayers];
};
// (masked = false: every entry is kept, for plain correlations such as the flow step's sums over pixels)
int launch_dw_reduce_blocks(const float *part, int nparts, float *dw, const DwBlocks &blocks, int Ctot, int k,
                            int pstride, hipStream_t stream, float sign = -1.0f, bool masked = true);
int launch_logdet_layers(const float *const *w, int layers, int C, int H, int W, int k, float *out,
                         hipStream_t stream);
struct ChainArgs {
    const float *in0;                    // input of stage 0
    const float *w[kChainMaxLayers];     // kernel of stage s
    float *out[kChainMaxLayers];         // output of stage s = input of stage s+1
    const float *map[kChainMaxLayers];   // flow step: affine channel map of stage s (C*C floats A, C floats d), or null
    int *flags;                          // progress counters (chain_flag_ints() ints)
    int *err;                            // error word (may be null): set to 1 when a bounded wait ran out
    int spin_limit;                      // set by launch_chain
    int stages, B, H, W, NB;
};
bool chain_supported(int stages, int C, int H, int W, int k);
bool chain_single_preferred(int B, int C, int H);
size_t chain_flag_ints(int stages, int B);
int launch_chain(int dir, ChainArgs args, int C, int k, hipStream_t stream);
// y = M x (dir 0) or y = M^T x (dir 1) for the masked causal convolution M
int launch_conv(int dir, const float *x, const float *w, float *y, int B, int C, int H, int W, int k,
                hipStream_t stream);
// bf16 storage of the activations (fp32 arithmetic)
bool wave_tile_bf16_supported(int C, int H, int W, int k);
int launch_solve_wave_tile_bf16(int dir, const void *in, const float *w, void *out, int B, int C, int H, int W, int k,
                                hipStream_t stream);
int launch_bwd_wave_tile_bf16(const void *x, const float *w, const void *g, void *v, float *part, int B, int C, int H,
                              int W, int k, hipStream_t stream);
int launch_bf16_to_f32(const void *in, float *out, size_t n, hipStream_t stream);
int launch_f32_to_bf16(const float *in, void *out, size_t n, hipStream_t stream);
bool conv_bwd_fused_supported(int C, int H, int W, int k);
size_t conv_bwd_fused_rows();
int launch_conv_bwd_fused(const float *g, const float *w, float *dx, const float *x, float *part, int B, int C, int H,
                          int W, int k, hipStream_t stream, unsigned *rows);
int launch_logdet(const float *w, int C, int H, int W, int k, float *out, hipStream_t stream);

// One flow step (inverse convolution, per-channel affine map, 1 x 1 convolution): invconv_flow.hip
size_t flow_mats_floats(int C);
bool flow_fused_supported(int C, int H, int W, int k);
bool flow_fused_preferred(int B, int C, int H, int W);
size_t flow_stat_rows(int B, int HW);
int launch_flow_prep(const float *w, const float *s, const float *b, const float *Q, float *mats, float *logdet, int C,
                     int H, int W, int k, hipStream_t stream);
// out[n][o][p] = add[o] + sum_i M[o][i] in[n][i][p] (transposed: M[i][o]); add may be null
int launch_flow_affine(bool transposed, const float *in, const float *M, const float *add, float *out, int B, int C,
                       int HW, hipStream_t stream);
int launch_flow_stats(const float *gz, const float *x, float *rows, int B, int C, int HW, hipStream_t stream);
int launch_rows_sum(const float *rows, int nrows, int stride, int E, float *out, hipStream_t stream);
bool flow_bwd_maps_supported(int C);
int launch_flow_bwd_maps(const float *z, const float *gz, const float *mats, float *x, float *g, float *rows, int B,
                         int C, int HW, hipStream_t stream);
int launch_flow_plane_sum(const float *gz, float *out, int planes, int HW, hipStream_t stream);
int launch_flow_finish(const float *sums, int have_dw, const float *w, const float *s, const float *b, const float *Q,
                       const float *mats, float *dLdw, float *dLds, float *dLdb, float *dLdQ, float lw, int C, int H,
                       int W, int k, hipStream_t stream);
int launch_flow_fwd_tile(const float *y, const float *w, const float *mats, float *z, int B, int C, int H, int W, int k,
                         hipStream_t stream);
int launch_flow_bwd_tile(const float *z, const float *w, const float *gz, const float *mats, float *v, float *part,
                         int B, int C, int H, int W, int k, hipStream_t stream);

}  // namespace invconv
