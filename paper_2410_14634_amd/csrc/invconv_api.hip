// C ABI of the inverse-convolution library: argument validation and dispatch.
#include <mutex>

#include "invconv_launch.h"

namespace invconv {

size_t solve_ws_bytes(int B, int C, int H, int W, int k)
{
    // only the few-channel images of more than 64 rows have a kernel that spreads one image over workgroups
    if (!wave_supported(C, H, k) && wave_bands_supported(C, H, W, k))
        return wave_bands_ws_bytes(B, C, H, W, k);
    // many channels with a kernel size other than 3: the folded weights of the call
    if (wide_stream_supported(C, H, k))
        return wide_stream_ws_bytes(C, k);
    // many channels, 3 x 3: the same, so that the weights are folded once per call and not once per workgroup
    return wide_prefold_ws_bytes(C, H, k);
}

}  // namespace invconv

using namespace invconv;

namespace {

constexpr int kVersion = 100;   // 0.1.0

int check_shape(int B, int C, int H, int W, int k)
{
    if (B < 1 || C < 1 || H < 1 || W < 1 || k < 1)
        return INVCONV_ERR_SHAPE;
    const long long lim = 0x7fffffffLL;
    if ((long long)B * C * H * W > lim || (long long)C * C * k * k > lim || (long long)H + W > lim)
        return INVCONV_ERR_SHAPE;
    // the kernels address inside one image with 32-bit byte offsets
    if ((long long)C * H * W >= (1LL << 29))
        return INVCONV_ERR_SHAPE;
    return INVCONV_OK;
}

int check_supported(int C, int H, int k)
{
    return solve_block_lds_bytes(C, H, k) <= kMaxLdsBytes ? INVCONV_OK : INVCONV_ERR_UNSUPPORTED;
}

constexpr size_t kWsHeader = INVCONV_WS_HEADER_BYTES;
size_t up256(size_t v) { return (v + 255) / 256 * 256; }

// Workspace of invconv_fwd_ws: header, then what the solve can use.
// Workspace of invconv_bwd / invconv_conv_bwd: header, the solve's share, then the partial sums of dL/dw.
struct WsLayout {
    size_t solve_bytes, dw_off, dw_bytes, total;
};

bool ws_layout(int B, int C, int H, int W, int k, bool with_dw, WsLayout *lay)
{
    lay->solve_bytes = up256(solve_ws_bytes(B, C, H, W, k));
    lay->dw_off = kWsHeader + lay->solve_bytes;
    lay->dw_bytes = 0;
    if (with_dw) {
        const DwPlan p = plan_dw_any(B, C, H, W, k);
        if (!p.rt)
            return false;
        lay->dw_bytes = up256(p.bytes);
        // the fused backward of the convolution itself writes one row per workgroup
        if (conv_bwd_fused_supported(C, H, W, k)) {
            const size_t rows = up256(conv_bwd_fused_rows() * (size_t)C * C * k * k * sizeof(float));
            lay->dw_bytes = lay->dw_bytes > rows ? lay->dw_bytes : rows;
        }
    }
    lay->total = lay->dw_off + lay->dw_bytes;
    return true;
}

SolveWs solve_ws_of(void *workspace, const WsLayout &lay)
{
    SolveWs ws;
    if (workspace) {
        ws.base = (char *)workspace + kWsHeader;
        ws.bytes = lay.solve_bytes;
        ws.err = (int *)((char *)workspace + INVCONV_WS_ERROR_WORD_OFFSET);
    }
    return ws;
}

int solve_variant(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W, int k,
                  hipStream_t stream, int variant, SolveWs ws);

// `logdet` (forward direction only, may be null): where log|det dx/dy| of one image goes; the few-channel, band and
// many-channel kernels write it on the side, every other kernel is followed by the small launch invconv_logdet makes.
// the caller's scratch as the place for the folded weights of a many-channel 3 x 3 solve, if it is large enough
float *wide_gw(const SolveWs &ws, int C, int H, int k)
{
    const size_t need = wide_prefold_ws_bytes(C, H, k);
    return need && ws.base && ws.bytes >= need ? reinterpret_cast<float *>(ws.base) : nullptr;
}

int solve(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W, int k,
          hipStream_t stream, int variant, SolveWs ws = SolveWs{}, float *logdet = nullptr)
{
    if (variant == INVCONV_VARIANT_AUTO && wave_supported(C, H, k))
        return wave_split_preferred(B, H, W, k) && !wave_tile_preferred(B, C, H, W)
                   ? launch_solve_wave_split(dir, in, w, out, B, C, H, W, k, stream, logdet)
                   : launch_solve_wave(dir, in, w, out, B, C, H, W, k, stream, logdet);
    // the band and many-channel kernels have a wave to spare for it too
    if (variant == INVCONV_VARIANT_AUTO && logdet && !wave_bands_supported(C, H, W, k)) {
        if (band_supported(C, H, k)) {
            if (!(chain_supported(1, C, H, W, k) && chain_single_preferred(B, C, H)))
                return launch_solve_band(dir, in, w, out, B, C, H, W, k, stream, logdet);
        } else if (wide_supported(C, H, k)) {
            return launch_solve_wide(dir, in, w, out, B, C, H, W, k, stream, logdet, wide_gw(ws, C, H, k));
        }
    }
    if (int s = solve_variant(dir, in, w, out, B, C, H, W, k, stream, variant, ws))
        return s;
    return logdet ? launch_logdet(w, C, H, W, k, logdet, stream) : INVCONV_OK;
}

int solve_variant(int dir, const float *in, const float *w, float *out, int B, int C, int H, int W, int k,
                  hipStream_t stream, int variant, SolveWs ws)
{
    switch (variant) {
    case INVCONV_VARIANT_AUTO:
        if (wave_supported(C, H, k))
            return wave_split_preferred(B, H, W, k) && !wave_tile_preferred(B, C, H, W)
                       ? launch_solve_wave_split(dir, in, w, out, B, C, H, W, k, stream)
                       : launch_solve_wave(dir, in, w, out, B, C, H, W, k, stream);
        if (wave_bands_supported(C, H, W, k))
            return launch_solve_wave_bands(dir, in, w, out, B, C, H, W, k, stream, ws);
        if (band_supported(C, H, k)) {
            if (chain_supported(1, C, H, W, k) && chain_single_preferred(B, C, H)) {
                ChainArgs a{};          // the pipelined kernel with one stage: no counters, no workspace
                a.in0 = in;
                a.w[0] = w;
                a.out[0] = out;
                a.stages = 1;
                a.B = B;
                a.H = H;
                a.W = W;
                return launch_chain(dir, a, C, k, stream);
            }
            return launch_solve_band(dir, in, w, out, B, C, H, W, k, stream);
        }
        if (wide_supported(C, H, k))
            return launch_solve_wide(dir, in, w, out, B, C, H, W, k, stream, nullptr, wide_gw(ws, C, H, k));
        if (wide_stream_supported(C, H, k) && ws.base && ws.bytes >= wide_stream_ws_bytes(C, k))
            return launch_solve_wide_stream(dir, in, w, out, B, C, H, W, k, stream, reinterpret_cast<float *>(ws.base));
        if (check_supported(C, H, k) == INVCONV_OK)
            return launch_solve_block(dir, in, w, out, B, C, H, W, k, stream);
        // nothing on chip holds this shape (more than 48 channels, or a window that outgrows LDS): one launch per
        // anti-diagonal with the kernel read from memory - slow, but nearly every shape has a solve
        return launch_solve_diag_wave(dir, in, w, out, B, C, H, W, k, stream);
    case INVCONV_VARIANT_BLOCK:
        return launch_solve_block(dir, in, w, out, B, C, H, W, k, stream);
    case INVCONV_VARIANT_WAVE:
        if (wave_bands_supported(C, H, W, k))
            return launch_solve_wave_bands(dir, in, w, out, B, C, H, W, k, stream, ws);
        return launch_solve_wave(dir, in, w, out, B, C, H, W, k, stream);
    case INVCONV_VARIANT_BAND:
        return launch_solve_band(dir, in, w, out, B, C, H, W, k, stream);
    case INVCONV_VARIANT_PERSISTENT:
        return launch_solve_persistent(dir, in, w, out, B, C, H, W, k, stream);
    case INVCONV_VARIANT_WAVE_SPLIT:
        return launch_solve_wave_split(dir, in, w, out, B, C, H, W, k, stream);
    case INVCONV_VARIANT_DIAG_LAUNCH:
        return launch_solve_diag(dir, in, w, out, B, C, H, W, k, stream);
    default:
        return INVCONV_ERR_VARIANT;
    }
}

int fwd_impl(const float *y, const float *w, float *x, int B, int C, int H, int W, int k, void *stream, int variant,
             SolveWs ws, float *logdet = nullptr)
{
    if (!y || !w || !x)
        return INVCONV_ERR_NULL;
    if (int s = check_shape(B, C, H, W, k))
        return s;
    if (x == y || (const float *)x == w)
        return INVCONV_ERR_ALIAS;
    if (variant < INVCONV_VARIANT_AUTO || variant > INVCONV_VARIANT_WAVE_SPLIT)
        return INVCONV_ERR_VARIANT;
    if (variant == INVCONV_VARIANT_WAVE_SPLIT && !wave_supported(C, H, k))
        return INVCONV_ERR_VARIANT;
    if (variant == INVCONV_VARIANT_WAVE && !wave_supported(C, H, k) && !wave_bands_supported(C, H, W, k))
        return INVCONV_ERR_VARIANT;
    if (variant == INVCONV_VARIANT_BAND && !band_supported(C, H, k))
        return INVCONV_ERR_VARIANT;
    if (variant == INVCONV_VARIANT_BLOCK)
        if (int s = check_supported(C, H, k))
            return s;
    return solve(0, y, w, x, B, C, H, W, k, (hipStream_t)stream, variant, ws, logdet);
}

}  // namespace

extern "C" {

invconv_status invconv_fwd_ex(const float *y, const float *w, float *x, int B, int C, int H, int W, int k,
                              void *stream, int variant)
{
    return fwd_impl(y, w, x, B, C, H, W, k, stream, variant, SolveWs{});
}

invconv_status invconv_fwd(const float *y, const float *w, float *x, int B, int C, int H, int W, int k,
                           void *stream)
{
    return fwd_impl(y, w, x, B, C, H, W, k, stream, INVCONV_VARIANT_AUTO, SolveWs{});
}

invconv_status invconv_fwd_logdet(const float *y, const float *w, float *x, float *logdet, int B, int C, int H, int W,
                                  int k, void *stream)
{
    if (!logdet)
        return INVCONV_ERR_NULL;
    if ((const float *)logdet == y || (const float *)logdet == w || logdet == x)
        return INVCONV_ERR_ALIAS;
    return fwd_impl(y, w, x, B, C, H, W, k, stream, INVCONV_VARIANT_AUTO, SolveWs{}, logdet);
}

size_t invconv_fwd_workspace_bytes(int B, int C, int H, int W, int k)
{
    WsLayout lay;
    if (check_shape(B, C, H, W, k) != INVCONV_OK || !ws_layout(B, C, H, W, k, false, &lay))
        return 0;
    return lay.total;
}

invconv_status invconv_fwd_ws(const float *y, const float *w, float *x, int B, int C, int H, int W, int k,
                              void *workspace, size_t workspace_bytes, void *stream)
{
    if (!y || !w || !x)
        return INVCONV_ERR_NULL;
    if (int s = check_shape(B, C, H, W, k))
        return s;
    WsLayout lay;
    ws_layout(B, C, H, W, k, false, &lay);
    if (!workspace || workspace_bytes < lay.total || ((size_t)workspace & 255))
        return INVCONV_ERR_WORKSPACE;
    return fwd_impl(y, w, x, B, C, H, W, k, stream, INVCONV_VARIANT_AUTO, solve_ws_of(workspace, lay));
}

void invconv_set_wait_budget(int polls) { set_wait_budget(polls); }

invconv_status invconv_workspace_error(const void *workspace, void *stream, int *word)
{
    if (!workspace || !word)
        return INVCONV_ERR_NULL;
    if (hipMemcpyAsync(word, (const char *)workspace + INVCONV_WS_ERROR_WORD_OFFSET, sizeof(int), hipMemcpyDeviceToHost,
                       (hipStream_t)stream) != hipSuccess ||
        hipStreamSynchronize((hipStream_t)stream) != hipSuccess) {
        (void)hipGetLastError();
        return INVCONV_ERR_LAUNCH;
    }
    return INVCONV_OK;
}

invconv_status invconv_conv_fwd(const float *x, const float *w, float *y, int B, int C, int H, int W, int k,
                                void *stream)
{
    if (!x || !w || !y)
        return INVCONV_ERR_NULL;
    if (int s = check_shape(B, C, H, W, k))
        return s;
    if (y == x || (const float *)y == w)
        return INVCONV_ERR_ALIAS;
    return launch_conv(0, x, w, y, B, C, H, W, k, (hipStream_t)stream);
}

invconv_status invconv_conv_bwd(const float *x, const float *w, const float *dLdy, float *dLdx, float *dLdw, int B,
                                int C, int H, int W, int k, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!x || !w || !dLdy || !dLdx || !dLdw)
        return INVCONV_ERR_NULL;
    if (int s = check_shape(B, C, H, W, k))
        return s;
    if (dLdx == dLdy || dLdx == x || (const float *)dLdx == w || dLdw == dLdx || (const float *)dLdw == w ||
        (const float *)dLdw == x || (const float *)dLdw == dLdy)
        return INVCONV_ERR_ALIAS;
    const DwPlan p = plan_dw_any(B, C, H, W, k);
    WsLayout lay;
    if (!p.rt || !ws_layout(B, C, H, W, k, true, &lay))
        return INVCONV_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < lay.total || ((size_t)workspace & 255))
        return INVCONV_ERR_WORKSPACE;
    float *part = (float *)((char *)workspace + lay.dw_off);
    hipStream_t st = (hipStream_t)stream;
    if (conv_bwd_fused_supported(C, H, W, k) && ((((size_t)x | (size_t)dLdy | (size_t)dLdx)) & 15) == 0) {
        unsigned rows = 0;
        if (int s = launch_conv_bwd_fused(dLdy, w, dLdx, x, part, B, C, H, W, k, st, &rows))
            return s;
        return launch_dw_reduce(part, (int)rows, dLdw, C, k, st, 1.0f);
    }
    if (int s = launch_conv(1, dLdy, w, dLdx, B, C, H, W, k, st))
        return s;
    if (dw_mfma_supported(C, k) && plan_dw_mfma(B, C, H, W, k).rt)
        return launch_dw_mfma(x, dLdy, dLdw, part, p, B, C, H, W, k, st, 1.0f);
    return launch_dw(x, dLdy, dLdw, part, p, B, C, H, W, k, st, 1.0f);
}

size_t invconv_bwd_workspace_bytes(int B, int C, int H, int W, int k)
{
    WsLayout lay;
    if (check_shape(B, C, H, W, k) != INVCONV_OK || !ws_layout(B, C, H, W, k, true, &lay))
        return 0;
    return lay.total;
}

invconv_status invconv_bwd_ex(const float *x, const float *w, const float *dLdx, float *dLdy, float *dLdw,
                              int B, int C, int H, int W, int k, void *workspace, size_t workspace_bytes,
                              void *stream, int variant)
{
    if (!x || !w || !dLdx || !dLdy || !dLdw)
        return INVCONV_ERR_NULL;
    if (int s = check_shape(B, C, H, W, k))
        return s;
    if (dLdy == dLdx || dLdy == x || (const float *)dLdy == w || dLdw == dLdy || (const float *)dLdw == w ||
        (const float *)dLdw == x || (const float *)dLdw == dLdx)
        return INVCONV_ERR_ALIAS;
    if (variant < INVCONV_VARIANT_AUTO || variant > INVCONV_VARIANT_WAVE_SPLIT)
        return INVCONV_ERR_VARIANT;
    if (variant == INVCONV_VARIANT_WAVE_SPLIT && !wave_supported(C, H, k))
        return INVCONV_ERR_VARIANT;
    if (variant == INVCONV_VARIANT_WAVE && !wave_supported(C, H, k) && !wave_bands_supported(C, H, W, k))
        return INVCONV_ERR_VARIANT;
    if (variant == INVCONV_VARIANT_BAND && !band_supported(C, H, k))
        return INVCONV_ERR_VARIANT;
    if (variant == INVCONV_VARIANT_BLOCK)
        if (int s = check_supported(C, H, k))
            return s;
    const DwPlan p = plan_dw_any(B, C, H, W, k);
    WsLayout lay;
    if (!p.rt || !ws_layout(B, C, H, W, k, true, &lay))
        return INVCONV_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < lay.total || ((size_t)workspace & 255))
        return INVCONV_ERR_WORKSPACE;
    float *part = (float *)((char *)workspace + lay.dw_off);
    hipStream_t st = (hipStream_t)stream;
    const bool separate = variant == INVCONV_VARIANT_AUTO && !bwd_wave_fused_pays(B, C, H, W, k) &&
                          conv_bwd_fused_supported(C, H, W, k) && ((((size_t)x | (size_t)dLdy)) & 15) == 0;
    if (!separate && (variant == INVCONV_VARIANT_AUTO || variant == INVCONV_VARIANT_WAVE) &&
        bwd_wave_supported(C, H, W, k)) {
        if (int s = launch_bwd_wave(x, w, dLdx, dLdy, part, B, C, H, W, k, st))
            return s;
        return launch_dw_reduce(part, B, dLdw, C, k, st);
    }
    if (int s = solve(1, dLdx, w, dLdy, B, C, H, W, k, st, variant, solve_ws_of(workspace, lay)))
        return s;
    if (conv_bwd_fused_supported(C, H, W, k) && ((((size_t)x | (size_t)dLdy)) & 15) == 0) {
        // few channels (tall images, large kernels): Theorem 2's sums as 4x4x1 outer products, x and dL/dy read once
        unsigned rows = 0;
        if (int s = launch_conv_bwd_fused(dLdy, w, nullptr, x, part, B, C, H, W, k, st, &rows))
            return s;
        return launch_dw_reduce(part, (int)rows, dLdw, C, k, st);
    }
    if (dw_mfma_supported(C, k) && plan_dw_mfma(B, C, H, W, k).rt)
        return launch_dw_mfma(x, dLdy, dLdw, part, p, B, C, H, W, k, st);
    return launch_dw(x, dLdy, dLdw, part, p, B, C, H, W, k, st);
}

invconv_status invconv_bwd(const float *x, const float *w, const float *dLdx, float *dLdy, float *dLdw, int B,
                           int C, int H, int W, int k, void *workspace, size_t workspace_bytes, void *stream)
{
    return invconv_bwd_ex(x, w, dLdx, dLdy, dLdw, B, C, H, W, k, workspace, workspace_bytes, stream,
                          INVCONV_VARIANT_AUTO);
}

}  // extern "C"

// ---------------------------------------------------------------------------
// Scratch of the entry point that takes no workspace (for callers that cannot allocate): one array in
// every device's memory for as long as the library is loaded.  In host code its name only stands for
// the symbol; the address in a device's memory comes from hipGetSymbolAddress, asked once per device
// with that device current, and only that address is ever handed to a kernel.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[INVCONV_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];       // [device] address of that device's copy of `scratch`
std::mutex g_scratch_mutex;

int static_scratch(void **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return INVCONV_ERR_LAUNCH;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return INVCONV_ERR_LAUNCH;
        }
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return INVCONV_OK;
}

}  // namespace

extern "C" {

invconv_status invconv_bwd_static(const float *x, const float *w, const float *dLdx, float *dLdy, float *dLdw, int B,
                                  int C, int H, int W, int k, void *stream)
{
    if (!x || !w || !dLdx || !dLdy || !dLdw)
        return INVCONV_ERR_NULL;
    if (int s = check_shape(B, C, H, W, k))
        return s;
    const size_t need = invconv_bwd_workspace_bytes(B, C, H, W, k);
    if (!need)
        return INVCONV_ERR_UNSUPPORTED;
    if (need > (size_t)INVCONV_STATIC_SCRATCH_BYTES)
        return INVCONV_ERR_WORKSPACE;       // this shape needs more scratch than the library holds
    void *ws = nullptr;
    if (int s = static_scratch(&ws))
        return s;
    return invconv_bwd(x, w, dLdx, dLdy, dLdw, B, C, H, W, k, ws, INVCONV_STATIC_SCRATCH_BYTES, stream);
}

// ---- bf16 storage variant: activations as bf16 in memory, fp32 arithmetic ----
size_t invconv_bf16_workspace_bytes(int B, int C, int H, int W, int k)
{
    WsLayout lay;
    if (check_shape(B, C, H, W, k) != INVCONV_OK || !ws_layout(B, C, H, W, k, true, &lay))
        return 0;
    return lay.total + 3 * up256((size_t)B * C * H * W * sizeof(float));     // fp32 copies for shapes without a bf16 kernel
}

invconv_status invconv_fwd_bf16(const void *y, const float *w, void *x, int B, int C, int H, int W, int k,
                                void *workspace, size_t workspace_bytes, void *stream)
{
    if (!y || !w || !x)
        return INVCONV_ERR_NULL;
    if (int s = check_shape(B, C, H, W, k))
        return s;
    if (x == y || x == (const void *)w)
        return INVCONV_ERR_ALIAS;
    WsLayout lay;
    if (!ws_layout(B, C, H, W, k, true, &lay))
        return INVCONV_ERR_UNSUPPORTED;
    const size_t act = up256((size_t)B * C * H * W * sizeof(float));
    if (!workspace || workspace_bytes < lay.total + 3 * act || ((size_t)workspace & 255))
        return INVCONV_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    if (wave_tile_bf16_supported(C, H, W, k) && ((((size_t)y | (size_t)x)) & 7) == 0)
        return launch_solve_wave_tile_bf16(0, y, w, x, B, C, H, W, k, st);
    float *t0 = (float *)((char *)workspace + lay.total), *t1 = (float *)((char *)workspace + lay.total + act);
    const size_t n = (size_t)B * C * H * W;
    if (int s = launch_bf16_to_f32(y, t0, n, st))
        return s;
    if (int s = fwd_impl(t0, w, t1, B, C, H, W, k, stream, INVCONV_VARIANT_AUTO, solve_ws_of(workspace, lay)))
        return s;
    return launch_f32_to_bf16(t1, x, n, st);
}

invconv_status invconv_bwd_bf16(const void *x, const float *w, const void *dLdx, void *dLdy, float *dLdw, int B, int C,
                                int H, int W, int k, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!x || !w || !dLdx || !dLdy || !dLdw)
        return INVCONV_ERR_NULL;
    if (int s = check_shape(B, C, H, W, k))
        return s;
    if (dLdy == dLdx || dLdy == x || dLdy == (const void *)w || (const void *)dLdw == dLdy || (const float *)dLdw == w ||
        (const void *)dLdw == x || (const void *)dLdw == dLdx)
        return INVCONV_ERR_ALIAS;
    WsLayout lay;
    if (!ws_layout(B, C, H, W, k, true, &lay))
        return INVCONV_ERR_UNSUPPORTED;
    const size_t act = up256((size_t)B * C * H * W * sizeof(float));
    if (!workspace || workspace_bytes < lay.total + 3 * act || ((size_t)workspace & 255))
        return INVCONV_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    char *ws = (char *)workspace;
    if (wave_tile_bf16_supported(C, H, W, k) && ((((size_t)x | (size_t)dLdx | (size_t)dLdy)) & 7) == 0) {
        float *part = (float *)(ws + lay.dw_off);
        if (int s = launch_bwd_wave_tile_bf16(x, w, dLdx, dLdy, part, B, C, H, W, k, st))
            return s;
        return launch_dw_reduce(part, B, dLdw, C, k, st);
    }
    float *t0 = (float *)(ws + lay.total), *t1 = (float *)(ws + lay.total + act), *t2 = (float *)(ws + lay.total + 2 * act);
    const size_t n = (size_t)B * C * H * W;
    if (int s = launch_bf16_to_f32(x, t0, n, st))
        return s;
    if (int s = launch_bf16_to_f32(dLdx, t1, n, st))
        return s;
    if (int s = invconv_bwd(t0, w, t1, t2, dLdw, B, C, H, W, k, workspace, lay.total, stream))
        return s;
    return launch_f32_to_bf16(t2, dLdy, n, st);
}

invconv_status invconv_logdet(const float *w, int C, int H, int W, int k, float *out, void *stream)
{
    if (!w || !out)
        return INVCONV_ERR_NULL;
    if (int s = check_shape(1, C, H, W, k))
        return s;
    return launch_logdet(w, C, H, W, k, out, (hipStream_t)stream);
}

namespace {

// Workspace of the flow-step calls: the workspace of invconv_bwd for the same shape first (so that the
// separate-pass form can hand its start to the backward pass of the inverse convolution, sharing the header),
// then the step's small matrices, the summed rows, the partial rows, and two activation-sized buffers for the
// separate-pass form (x recomputed from z, and A^T dL/dz).
struct FlowLayout {
    size_t bwd_bytes, mats_off, sums_off, rows_off, tmp_off, tmp_bytes, total;
};

bool flow_layout(int B, int C, int H, int W, int k, FlowLayout *lay)
{
    WsLayout bl;
    if (check_shape(B, C, H, W, k) != INVCONV_OK || !ws_layout(B, C, H, W, k, true, &bl))
        return false;
    const size_t P = (size_t)C * C * k * k, E2 = (size_t)C * C + C;
    lay->bwd_bytes = bl.total;
    lay->mats_off = bl.total;
    lay->sums_off = lay->mats_off + up256(flow_mats_floats(C) * sizeof(float));
    lay->rows_off = lay->sums_off + up256((P + E2) * sizeof(float));
    // partial rows: the fused few-channel kernel's [P | C*C | C] per image, or the generic sums' rows, or
    // (C <= 16) the partial sums of the matrix-core correlation with k = 1 followed by one value per plane
    size_t rows_bytes = (size_t)B * (P + E2) * sizeof(float);
    const size_t rows_sep = flow_stat_rows(B, H * W) * E2 * sizeof(float);
    rows_bytes = rows_bytes > rows_sep ? rows_bytes : rows_sep;
    const DwPlan p1 = plan_dw_any(B, C, H, W, 1);
    if (p1.rt) {
        const size_t with_planes = up256(p1.bytes) + (size_t)B * C * sizeof(float);
        rows_bytes = rows_bytes > with_planes ? rows_bytes : with_planes;
    }
    lay->tmp_off = lay->rows_off + up256(rows_bytes);
    lay->tmp_bytes = up256((size_t)B * C * H * W * sizeof(float));
    lay->total = lay->tmp_off + 2 * lay->tmp_bytes;
    return true;
}

// M2[o][i] = sum dLdz[o] x[i] and m1[o] = sum dLdz[o] over batch and pixels into sums = [C*C | C]
int flow_sums(const float *dLdz, const float *x, float *rows, float *sums, int B, int C, int H, int W, hipStream_t st)
{
    const int E2 = C * C + C;
    const DwPlan p1 = plan_dw_any(B, C, H, W, 1);
    if (dw_mfma_supported(C, 1) && p1.rt && !p1.cb && plan_dw_mfma(B, C, H, W, 1).rt) {
        // the correlation of Eq. 4 with a 1 x 1 window, neither negated nor masked, is exactly M2
        if (int rc = launch_dw_mfma_partial(x, dLdz, rows, p1, B, C, H, W, 1, st))
            return rc;
        if (int rc = launch_rows_sum(rows, (int)p1.nparts, C * C, C * C, sums, st))
            return rc;
        float *planes = (float *)((char *)rows + up256(p1.bytes));
        if (int rc = launch_flow_plane_sum(dLdz, planes, B * C, H * W, st))
            return rc;
        return launch_rows_sum(planes, B, C, C, sums + (size_t)C * C, st);
    }
    if (dw_mfma_supported(C, 1) && p1.rt && p1.cb && plan_dw_mfma(B, C, H, W, 1).rt) {
        // more than 16 channels: the same correlation in blocks of channels, both passes, unmasked and un-negated
        if (int rc = launch_dw_mfma(x, dLdz, sums, rows, p1, B, C, H, W, 1, st, 1.0f, false))
            return rc;
        float *planes = (float *)((char *)rows + up256(p1.bytes));
        if (int rc = launch_flow_plane_sum(dLdz, planes, B * C, H * W, st))
            return rc;
        return launch_rows_sum(planes, B, C, C, sums + (size_t)C * C, st);
    }
    if (int rc = launch_flow_stats(dLdz, x, rows, B, C, H * W, st))
        return rc;
    return launch_rows_sum(rows, (int)flow_stat_rows(B, H * W), E2, E2, sums, st);
}

bool aligned16(const void *a, const void *b, const void *c = nullptr, const void *d = nullptr)
{
    return (((size_t)a | (size_t)b | (size_t)c | (size_t)d) & 15) == 0;
}

}  // namespace

extern "C" {

size_t invconv_flowstep_workspace_bytes(int B, int C, int H, int W, int k)
{
    FlowLayout lay;
    return flow_layout(B, C, H, W, k, &lay) ? lay.total : 0;
}

invconv_status invconv_flowstep_fwd(const float *y, const float *w, const float *s, const float *b, const float *Q,
                                    float *z, float *logdet, int B, int C, int H, int W, int k, void *workspace,
                                    size_t workspace_bytes, void *stream)
{
    return invconv_flowstep_fwd_ex(y, w, s, b, Q, z, logdet, B, C, H, W, k, workspace, workspace_bytes, stream,
                                   INVCONV_FLOW_AUTO);
}

invconv_status invconv_flowstep_fwd_ex(const float *y, const float *w, const float *s, const float *b, const float *Q,
                                       float *z, float *logdet, int B, int C, int H, int W, int k, void *workspace,
                                       size_t workspace_bytes, void *stream, int form)
{
    if (form < INVCONV_FLOW_AUTO || form > INVCONV_FLOW_FUSED)
        return INVCONV_ERR_VARIANT;
    if (!y || !w || !s || !b || !Q || !z)
        return INVCONV_ERR_NULL;
    if (int st = check_shape(B, C, H, W, k))
        return st;
    if (z == y || (const float *)z == w || (const float *)z == s || (const float *)z == b || (const float *)z == Q ||
        (logdet && (logdet == z || (const float *)logdet == y)))
        return INVCONV_ERR_ALIAS;
    FlowLayout lay;
    if (!flow_layout(B, C, H, W, k, &lay))
        return INVCONV_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < lay.total || ((size_t)workspace & 255))
        return INVCONV_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    char *ws = (char *)workspace;
    float *mats = (float *)(ws + lay.mats_off);
    // few channels, few images: one launch, the split solve with the channel map on its way out
    if (form == INVCONV_FLOW_AUTO && flow_split_supported(B, C, H, W, k))
        return launch_flow_fwd_split(y, w, s, b, Q, z, B, C, H, W, k, st, logdet);
    // 5-16 channels on images of one band: the same on the one-band kernel
    if (form == INVCONV_FLOW_AUTO && flow_band_supported(C, H, k))
        return launch_flow_fwd_band(y, w, s, b, Q, z, B, C, H, W, k, st, logdet);
    if (int rc = launch_flow_prep(w, s, b, Q, mats, logdet, C, H, W, k, st))
        return rc;
    if (form != INVCONV_FLOW_SEPARATE && flow_fused_supported(C, H, W, k) && aligned16(y, z) &&
        (form == INVCONV_FLOW_FUSED || flow_fused_preferred(B, C, H, W)))
        return launch_flow_fwd_tile(y, w, mats, z, B, C, H, W, k, st);
    if (form != INVCONV_FLOW_SEPARATE && chain_supported(1, C, H, W, k) &&
        (form == INVCONV_FLOW_FUSED || chain_single_preferred(B, C, H))) {
        // 8-16 channels: the pipelined band kernel with the affine map applied by its storers
        ChainArgs a{};
        a.in0 = y;
        a.w[0] = w;
        a.out[0] = z;
        a.map[0] = mats;
        a.stages = 1;
        a.B = B;
        a.H = H;
        a.W = W;
        return launch_chain(0, a, C, k, st);
    }
    // separate passes: the solve into scratch, then the affine channel map
    float *x = (float *)(ws + lay.tmp_off);
    WsLayout bl;
    ws_layout(B, C, H, W, k, true, &bl);
    if (int rc = fwd_impl(y, w, x, B, C, H, W, k, stream, INVCONV_VARIANT_AUTO, solve_ws_of(workspace, bl)))
        return rc;
    return launch_flow_affine(false, x, mats, mats + (size_t)C * C, z, B, C, H * W, st);
}

invconv_status invconv_flowstep_bwd(const float *z, const float *w, const float *s, const float *b, const float *Q,
                                    const float *dLdz, float *dLdy, float *dLdw, float *dLds, float *dLdb,
                                    float *dLdQ, float logdet_weight, int B, int C, int H, int W, int k,
                                    void *workspace, size_t workspace_bytes, void *stream)
{
    return invconv_flowstep_bwd_ex(z, w, s, b, Q, dLdz, dLdy, dLdw, dLds, dLdb, dLdQ, logdet_weight, B, C, H, W, k,
                                   workspace, workspace_bytes, stream, INVCONV_FLOW_AUTO);
}

invconv_status invconv_flowstep_bwd_ex(const float *z, const float *w, const float *s, const float *b, const float *Q,
                                       const float *dLdz, float *dLdy, float *dLdw, float *dLds, float *dLdb,
                                       float *dLdQ, float logdet_weight, int B, int C, int H, int W, int k,
                                       void *workspace, size_t workspace_bytes, void *stream, int form)
{
    if (form < INVCONV_FLOW_AUTO || form > INVCONV_FLOW_FUSED)
        return INVCONV_ERR_VARIANT;
    if (!z || !w || !s || !b || !Q || !dLdz || !dLdy || !dLdw || !dLds || !dLdb || !dLdQ)
        return INVCONV_ERR_NULL;
    if (int st = check_shape(B, C, H, W, k))
        return st;
    const float *ins[] = {z, w, s, b, Q, dLdz};
    float *outs[] = {dLdy, dLdw, dLds, dLdb, dLdQ};
    for (float *o : outs) {
        for (const float *i : ins)
            if ((const float *)o == i)
                return INVCONV_ERR_ALIAS;
    }
    for (int a = 0; a < 5; ++a)
        for (int c = a + 1; c < 5; ++c)
            if (outs[a] == outs[c])
                return INVCONV_ERR_ALIAS;
    FlowLayout lay;
    if (!flow_layout(B, C, H, W, k, &lay))
        return INVCONV_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < lay.total || ((size_t)workspace & 255))
        return INVCONV_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    char *ws = (char *)workspace;
    float *mats = (float *)(ws + lay.mats_off), *sums = (float *)(ws + lay.sums_off), *rows = (float *)(ws + lay.rows_off);
    const int P = C * C * k * k, E2 = C * C + C;
    // few channels, few images: two launches, the eight-wave backward kernel with the channel maps inside and the
    // kernel that sums its rows and finishes the parameter gradients
    if (form == INVCONV_FLOW_AUTO && flow_bwd_split_supported(B, C, H, W, k)) {
        if (int rc = launch_flow_bwd_split(z, w, dLdz, s, b, Q, dLdy, rows, B, C, H, W, k, st))
            return rc;
        return launch_flow_finish_rows(rows, B, w, s, b, Q, dLdw, dLds, dLdb, dLdQ, logdet_weight, C, H, W, k, st);
    }
    if (int rc = launch_flow_prep(w, s, b, Q, mats, nullptr, C, H, W, k, st))
        return rc;
    if (form != INVCONV_FLOW_SEPARATE && flow_fused_supported(C, H, W, k) && aligned16(z, dLdz, dLdy) &&
        (form == INVCONV_FLOW_FUSED || flow_fused_preferred(B, C, H, W))) {
        if (int rc = launch_flow_bwd_tile(z, w, dLdz, mats, dLdy, rows, B, C, H, W, k, st))
            return rc;
        if (int rc = launch_rows_sum(rows, B, P + E2, P + E2, sums, st))
            return rc;
        return launch_flow_finish(sums, 1, w, s, b, Q, mats, dLdw, dLds, dLdb, dLdQ, logdet_weight, C, H, W, k, st);
    }
    float *x = (float *)(ws + lay.tmp_off), *g = (float *)(ws + lay.tmp_off + lay.tmp_bytes);
    const size_t CC = (size_t)C * C;
    if (form != INVCONV_FLOW_SEPARATE && chain_supported(1, C, H, W, k) &&
        (form == INVCONV_FLOW_FUSED || chain_single_preferred(B, C, H))) {
        // 8-16 channels: the transposed solve in the pipelined band kernel with A^T folded into its input
        // weights (dL/dz in, dL/dy out); x is recomputed once into scratch for the two sums over pixels
        ChainArgs a{};
        a.in0 = dLdz;
        a.w[0] = w;
        a.out[0] = dLdy;
        a.map[0] = mats;
        a.stages = 1;
        a.B = B;
        a.H = H;
        a.W = W;
        if (int rc = launch_chain(1, a, C, k, st))
            return rc;
        if (int rc = launch_flow_affine(false, z, mats + CC + C, mats + 2 * CC + C, x, B, C, H * W, st))
            return rc;
        WsLayout bl;
        ws_layout(B, C, H, W, k, true, &bl);
        const DwPlan p = plan_dw_any(B, C, H, W, k);
        float *part = (float *)(ws + bl.dw_off);
        if (dw_mfma_supported(C, k) && plan_dw_mfma(B, C, H, W, k).rt) {
            if (int rc = launch_dw_mfma(x, dLdy, dLdw, part, p, B, C, H, W, k, st))
                return rc;
        } else if (int rc = launch_dw(x, dLdy, dLdw, part, p, B, C, H, W, k, st)) {
            return rc;
        }
        if (int rc = flow_sums(dLdz, x, rows, sums, B, C, H, W, st))
            return rc;
        return launch_flow_finish(sums, 0, w, s, b, Q, mats, dLdw, dLds, dLdb, dLdQ, logdet_weight, C, H, W, k, st);
    }
    // separate passes: x = A^-1 z + e and g = A^T dL/dz into scratch, the backward pass of the inverse
    // convolution on them, the two sums of the neighbours' gradients, and the common last kernel
    if (flow_bwd_maps_supported(C) && (size_t)B * C * H * W <= ((size_t)1 << 20)) {
        // up to 4 MB of activations (where launches, not bytes, are what a pass costs): one pass over z and dL/dz
        // gives x, g and the partial sums of M2 and m1 together.  Beyond that the chunked kernel loses to the
        // separate passes (4096 x 3x32x32: 270 against 243 us)
        if (int rc = launch_flow_bwd_maps(z, dLdz, mats, x, g, rows, B, C, H * W, st))
            return rc;
        if (int rc = launch_rows_sum(rows, (int)flow_stat_rows(B, H * W), E2, E2, sums, st))
            return rc;
        if (int rc = invconv_bwd(x, w, g, dLdy, dLdw, B, C, H, W, k, workspace, lay.bwd_bytes, stream))
            return rc;
        return launch_flow_finish(sums, 0, w, s, b, Q, mats, dLdw, dLds, dLdb, dLdQ, logdet_weight, C, H, W, k, st);
    }
    if (int rc = launch_flow_affine(false, z, mats + CC + C, mats + 2 * CC + C, x, B, C, H * W, st))
        return rc;
    if (int rc = launch_flow_affine(true, dLdz, mats, nullptr, g, B, C, H * W, st))
        return rc;
    if (int rc = invconv_bwd(x, w, g, dLdy, dLdw, B, C, H, W, k, workspace, lay.bwd_bytes, stream))
        return rc;
    if (int rc = flow_sums(dLdz, x, rows, sums, B, C, H, W, st))
        return rc;
    return launch_flow_finish(sums, 0, w, s, b, Q, mats, dLdw, dLds, dLdb, dLdQ, logdet_weight, C, H, W, k, st);
}

}  // extern "C"

namespace {

struct ChainLayout {
    size_t flags_bytes, grad_bytes, dw_bytes, total;
};

bool chain_layout(int L, int B, int C, int H, int W, int k, ChainLayout *lay)
{
    if (L < 1 || L > kChainMaxLayers || check_shape(B, C, H, W, k) != INVCONV_OK)
        return false;
    const DwPlan p = plan_dw_any(B, C, H, W, k);
    if (!p.rt)
        return false;
    // header, progress counters, intermediate gradients, partial sums of dL/dw
    lay->flags_bytes = kWsHeader + up256(chain_flag_ints(L, B) * sizeof(int));
    lay->grad_bytes = up256((size_t)B * C * H * W * sizeof(float));
    lay->dw_bytes = up256(p.bytes) * (size_t)L;      // pass 1 of all layers runs as one launch
    lay->total = lay->flags_bytes + (size_t)(L > 1 ? L - 1 : 0) * lay->grad_bytes + lay->dw_bytes;
    return true;
}

}  // namespace

size_t invconv_chain_workspace_bytes(int L, int B, int C, int H, int W, int k)
{
    ChainLayout lay;
    return chain_layout(L, B, C, H, W, k, &lay) ? lay.total : 0;
}

invconv_status invconv_chain_fwd(const float *y, const float *const *w, float *const *x, int L, int B, int C, int H,
                                 int W, int k, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!y || !w || !x)
        return INVCONV_ERR_NULL;
    if (L < 1 || L > kChainMaxLayers)
        return INVCONV_ERR_SHAPE;
    if (int s = check_shape(B, C, H, W, k))
        return s;
    for (int l = 0; l < L; ++l) {
        if (!w[l] || !x[l])
            return INVCONV_ERR_NULL;
        if (x[l] == y)
            return INVCONV_ERR_ALIAS;
        for (int m = 0; m < l; ++m)
            if (x[m] == x[l])
                return INVCONV_ERR_ALIAS;
    }
    ChainLayout lay;
    if (!chain_layout(L, B, C, H, W, k, &lay))
        return INVCONV_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < lay.total || ((size_t)workspace & 255))
        return INVCONV_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    if (chain_supported(L, C, H, W, k)) {
        ChainArgs a{};
        a.in0 = y;
        for (int l = 0; l < L; ++l) {
            a.w[l] = w[l];
            a.out[l] = x[l];
        }
        a.flags = (int *)((char *)workspace + kWsHeader);
        a.err = (int *)((char *)workspace + INVCONV_WS_ERROR_WORD_OFFSET);
        a.stages = L;
        a.B = B;
        a.H = H;
        a.W = W;
        return launch_chain(0, a, C, k, st);
    }
    for (int l = 0; l < L; ++l)
        if (int s = invconv_fwd(l == 0 ? y : x[l - 1], w[l], x[l], B, C, H, W, k, stream))
            return s;
    return INVCONV_OK;
}

invconv_status invconv_chain_bwd(const float *const *x, const float *const *w, const float *dLdx_last,
                                 float *dLdy_first, float *const *dLdw, int L, int B, int C, int H, int W, int k,
                                 void *workspace, size_t workspace_bytes, void *stream)
{
    if (!x || !w || !dLdx_last || !dLdy_first || !dLdw)
        return INVCONV_ERR_NULL;
    if (L < 1 || L > kChainMaxLayers)
        return INVCONV_ERR_SHAPE;
    if (int s = check_shape(B, C, H, W, k))
        return s;
    for (int l = 0; l < L; ++l) {
        if (!w[l] || !x[l] || !dLdw[l])
            return INVCONV_ERR_NULL;
        if (x[l] == dLdy_first)
            return INVCONV_ERR_ALIAS;
    }
    if (dLdy_first == dLdx_last)
        return INVCONV_ERR_ALIAS;
    ChainLayout lay;
    if (!chain_layout(L, B, C, H, W, k, &lay))
        return INVCONV_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < lay.total || ((size_t)workspace & 255))
        return INVCONV_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    char *ws = (char *)workspace;
    // v[l] = dL/dy of layer l: v[0] is the caller's output, the others live in the workspace
    float *v[kChainMaxLayers];
    v[0] = dLdy_first;
    for (int l = 1; l < L; ++l)
        v[l] = (float *)(ws + lay.flags_bytes + (size_t)(l - 1) * lay.grad_bytes);
    float *part = (float *)(ws + lay.flags_bytes + (size_t)(L > 1 ? L - 1 : 0) * lay.grad_bytes);
    if (chain_supported(L, C, H, W, k)) {
        ChainArgs a{};
        a.in0 = dLdx_last;
        for (int s = 0; s < L; ++s) {       // stage s solves layer L-1-s
            a.w[s] = w[L - 1 - s];
            a.out[s] = v[L - 1 - s];
        }
        a.flags = (int *)((char *)workspace + kWsHeader);
        a.err = (int *)((char *)workspace + INVCONV_WS_ERROR_WORD_OFFSET);
        a.stages = L;
        a.B = B;
        a.H = H;
        a.W = W;
        if (int s = launch_chain(1, a, C, k, st))
            return s;
    } else {
        for (int l = L - 1; l >= 0; --l)
            if (int s = solve(1, l == L - 1 ? dLdx_last : v[l + 1], w[l], v[l], B, C, H, W, k, st, INVCONV_VARIANT_AUTO))
                return s;
    }
    const DwPlan p = plan_dw_any(B, C, H, W, k);
    const bool mfma = dw_mfma_supported(C, k) && plan_dw_mfma(B, C, H, W, k).rt;
    if (mfma && !p.cb)
        return launch_dw_mfma_layers(x, v, dLdw, L, part, plan_dw_mfma_layers(L, B, C, H, W, k), B, C, H, W, k, st);
    if (mfma) {         // more than 16 channels: the blocked form, layer by layer
        for (int l = 0; l < L; ++l)
            if (int s = launch_dw_mfma(x[l], v[l], dLdw[l], part, p, B, C, H, W, k, st))
                return s;
        return INVCONV_OK;
    }
    for (int l = 0; l < L; ++l) {
        if (int s = launch_dw(x[l], v[l], dLdw[l], part, p, B, C, H, W, k, st))
            return s;
    }
    return INVCONV_OK;
}

invconv_status invconv_probe_step_sync(int mode, int steps, int workgroups, void *stream)
{
    if (mode < 0 || mode > 2)
        return INVCONV_ERR_VARIANT;
    if (steps < 1 || steps > 100000 || workgroups < 1 || workgroups > 256)
        return INVCONV_ERR_SHAPE;
    return launch_probe(mode, steps, workgroups, (hipStream_t)stream);
}

invconv_status invconv_chain_logdet(const float *const *w, int L, int C, int H, int W, int k, float *out,
                                    void *stream)
{
    if (!w || !out)
        return INVCONV_ERR_NULL;
    if (L < 1 || L > kChainMaxLayers)
        return INVCONV_ERR_SHAPE;
    if (int s = check_shape(1, C, H, W, k))
        return s;
    for (int l = 0; l < L; ++l)
        if (!w[l])
            return INVCONV_ERR_NULL;
    return launch_logdet_layers(w, L, C, H, W, k, out, (hipStream_t)stream);
}

const char *invconv_status_string(invconv_status status)
{
    switch (status) {
    case INVCONV_OK: return "ok";
    case INVCONV_ERR_NULL: return "null pointer argument";
    case INVCONV_ERR_SHAPE: return "invalid shape (a dimension < 1 or a size overflow)";
    case INVCONV_ERR_UNSUPPORTED: return "shape exceeds the kernels' on-chip buffers";
    case INVCONV_ERR_WORKSPACE: return "workspace missing or too small";
    case INVCONV_ERR_ALIAS: return "an output buffer aliases an input buffer";
    case INVCONV_ERR_LAUNCH: return "HIP kernel launch failed";
    case INVCONV_ERR_VARIANT: return "unknown or unavailable kernel variant";
    default: return "unknown status";
    }
}

int invconv_version(void) { return kVersion; }

}  // extern "C"
