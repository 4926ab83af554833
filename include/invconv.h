/*
 * invconv.h - C ABI of the MI355X (gfx950) inverse-convolution library.
 *
 * The operator is the inverse of a causally masked k x k convolution
 * (Section 3 of "Parallel Backpropagation for Inverse of a Convolution with
 * Application to Normalizing Flows"): the input image is zero-padded with k-1
 * rows on top and k-1 columns on the left, so output pixel (r,c) of
 * y = conv_w(x) reads x only at (r',c') with r-k < r' <= r, c-k < c' <= c, and
 * the bottom-right kernel tap multiplies the current pixel (Eq. 1).
 *
 * Conventions shared by every entry point
 *   - Every pointer except `stream` is a DEVICE pointer to contiguous fp32
 *     (unless a comment says HOST).  The caller owns all buffers; the library
 *     never allocates, frees or keeps device memory: all scratch comes in as
 *     `workspace` arguments (256-byte aligned device memory of at least the
 *     size the matching *_workspace_bytes() call returns), and the same
 *     kernels run whether or not the stream is being captured into a graph.
 *     `stream` is a hipStream_t (NULL = the default stream).  Calls are
 *     asynchronous on `stream`: no host synchronisation, no host read-back.
 *   - Workspace header.  The first INVCONV_WS_HEADER_BYTES bytes of every
 *     workspace belong to the library.  The int32 at byte offset
 *     INVCONV_WS_ERROR_WORD_OFFSET is the ERROR WORD.  Kernels that spread one
 *     image or one stack of layers over several workgroups order them with
 *     bounded waits; a wait that runs out (which a healthy device never
 *     shows) makes the waiting wave carry on, every kernel still ends, the
 *     affected outputs are filled with NaN, and the error word is set to 1.
 *     The library only ever sets the word, it never clears it: zero the header
 *     once after allocating the workspace, then read the word (4 bytes, device
 *     to host, or invconv_workspace_error()) whenever a result is consumed.
 *   - Activations (y, x, dLdx, dLdy) are [B][C][H][W].
 *   - Kernels (w, dLdw) are [C_out = C][C_in = C][k][k] (Algorithm 1's
 *     K[c, k_c, ., .]).  Tap (a,b) multiplies x[., r-(k-1)+a, c-(k-1)+b].
 *   - At the current-pixel tap (a,b) = (k-1,k-1) the channel mixing is lower
 *     triangular: entries w[o][i][k-1][k-1] with i > o are IGNORED whatever
 *     they hold, and the matching dLdw entries are written as 0.  The diagonal
 *     w[c][c][k-1][k-1] must be non-zero (the paper fixes it to 1); a zero
 *     diagonal is not checked and yields IEEE inf/NaN.
 *   - H != W, k > min(H,W) and k = 1 are valid.
 *   - Return value: INVCONV_OK or a negative invconv_status.  Argument and
 *     shape errors (NULL, SHAPE, UNSUPPORTED, WORKSPACE, ALIAS, VARIANT) are
 *     found before anything is launched: no output has been touched.
 *     INVCONV_ERR_LAUNCH means the runtime refused a launch; kernels of the
 *     same call queued before it still run, so outputs are undefined.
 */
#ifndef INVCONV_H
#define INVCONV_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int invconv_status;

#define INVCONV_WS_HEADER_BYTES 256
#define INVCONV_WS_ERROR_WORD_OFFSET 0

enum {
    INVCONV_OK = 0,
    INVCONV_ERR_NULL = -1,        /* a required pointer is NULL */
    INVCONV_ERR_SHAPE = -2,       /* B, C, H, W or k < 1, B*C*H*W > 2^31 - 1, or one image C*H*W >= 2^29 elements (2 GiB) */
    INVCONV_ERR_UNSUPPORTED = -3, /* shape beyond what the kernels' on-chip buffers hold: a kernel variant asked for by name, the
                                     weight gradient's tiles, or - the default solve falls back to one launch per anti-diagonal
                                     for shapes no on-chip kernel holds, far slower - more than 8192 kernel entries C k k per
                                     output channel */
    INVCONV_ERR_WORKSPACE = -4,   /* workspace NULL, not 256-byte aligned, smaller than *_workspace_bytes(), or
                                     (entry point without a workspace argument) larger than the library's own */
    INVCONV_ERR_ALIAS = -5,       /* an output pointer equals an input pointer */
    INVCONV_ERR_LAUNCH = -6,      /* the HIP runtime refused a launch */
    INVCONV_ERR_VARIANT = -7      /* unknown variant, or variant not available for this shape */
};

/* Kernel variants (for measurement; INVCONV_VARIANT_AUTO is what the plain calls use). */
enum {
    INVCONV_VARIANT_AUTO = 0,
    INVCONV_VARIANT_BLOCK = 1,    /* one workgroup per image, LDS window, one barrier per anti-diagonal */
    INVCONV_VARIANT_DIAG_LAUNCH = 2, /* one kernel launch per anti-diagonal (capture it in a hipGraph) */
    INVCONV_VARIANT_WAVE = 3,     /* one wave per 64 image rows, lane = row, register/DPP systolic solve (C <= 4 with k = 3, C = 3 also k = 2, 5, 7, 9, 11; H <= 512, k <= 5 beyond 64 rows; bands of one image hand over through LDS) */
    INVCONV_VARIANT_BAND = 4,     /* one wave per 16-row band, 16x16x4 MFMA systolic solve (C = 5 .. 16; k = 3 with H <= 128; k = 2, 5, 7 with H <= 64; k = 9, 11 at 8, 12, 16 channels with H <= 64) */
    INVCONV_VARIANT_PERSISTENT = 5, /* one cooperative launch, persistent grid, device-wide barrier per anti-diagonal */
    INVCONV_VARIANT_WAVE_SPLIT = 6 /* the wave solve with a step's matrix instructions split over four waves by the age of their input (same shapes, k >= 3, H <= 64) */
};

/*
 * Forward pass of the inverse convolution: solves conv_w(x) = y for x by
 * forward substitution, x_q = (y_q - sum_{r in Delta(q)} W_{(k,k)-q+r} x_r) / W_{k,k}
 * (Eq. 1 rearranged, as in the proofs of Theorems 1 and 2).  Pixels on one
 * anti-diagonal are independent and are processed in parallel; anti-diagonals
 * are processed in increasing order (Section 3.3).
 *   y [in]  B*C*H*W     w [in]  C*C*k*k     x [out] B*C*H*W, must not alias y.
 */
invconv_status invconv_fwd(const float *y, const float *w, float *x,
                           int B, int C, int H, int W, int k, void *stream);

/*
 * Forward pass and log-determinant in one call: what the forward pass of a flow step needs
 * (Section 4: the likelihood takes x and log|det dx/dy|).  x as invconv_fwd, *logdet as invconv_logdet;
 * for few-channel images (C <= 4, H <= 64) and for the band and many-channel kernels (8-48 channels)
 * both come out of one kernel launch.
 *   logdet [out] one device float.
 */
invconv_status invconv_fwd_logdet(const float *y, const float *w, float *x, float *logdet,
                                  int B, int C, int H, int W, int k, void *stream);

/*
 * The same forward pass with scratch from the caller.  Images of few channels (C <= 4) and more than
 * 64 rows are then cut into bands of 64 rows that run on different compute units and hand their
 * boundary messages over through the workspace (Section 3.3 only needs the pixels of an anti-diagonal
 * to be independent; a band trails the one above by a fixed number of steps); invconv_fwd, which has
 * nowhere to put those messages, keeps all bands of an image in one workgroup.  Images of 20 to 48
 * channels (multiples of 4) with a kernel size of 2, 5, 7, 9 or 11 keep the folded weights of the call
 * in the workspace and stream them to the matrix cores (invconv_fwd solves those one anti-diagonal per
 * launch, 15 to 30 times slower); with a 3 x 3 kernel the same channel counts fold their weights once
 * per call into the workspace instead of once per workgroup (100 images of 48 x 8 x 8: 53 -> 43 us,
 * 1024 images: 215 -> 123 us).  Other shapes run the kernels invconv_fwd runs.  Results agree to
 * rounding (the kernels add a pixel's terms in different orders).
 *   workspace [scratch] at least invconv_fwd_workspace_bytes() bytes (never 0 for a valid shape).
 */
invconv_status invconv_fwd_ws(const float *y, const float *w, float *x,
                              int B, int C, int H, int W, int k,
                              void *workspace, size_t workspace_bytes, void *stream);
size_t invconv_fwd_workspace_bytes(int B, int C, int H, int W, int k);   /* 0 if the shape is invalid */

/*
 * Reads the error word of a workspace: copies it to *word (HOST pointer) on `stream` and waits for the
 * stream.  0 = no bounded wait has run out since the header was last zeroed.
 */
invconv_status invconv_workspace_error(const void *workspace, void *stream, int *word);

/*
 * Test hook for the bounded waits: the number of polls a waiting wave makes before it gives up, for
 * all calls of this process from now on (0 = the built-in budgets, about a second).  With a budget of
 * a few polls the waits of a multi-workgroup kernel run out at once: outputs are NaN-filled, the error
 * word is set, every kernel still ends normally.
 */
void invconv_set_wait_budget(int polls);

/*
 * The masked causal convolution itself, y = conv_w(x) (Eq. 1): the inverse of invconv_fwd and the
 * only operator the sampling direction needs (Section 4.3).  Same layouts and masking conventions.
 *   x [in]  B*C*H*W     w [in]  C*C*k*k     y [out] B*C*H*W, must not alias x.
 */
invconv_status invconv_conv_fwd(const float *x, const float *w, float *y,
                                int B, int C, int H, int W, int k, void *stream);

/*
 * Gradients of that convolution (y = M x is linear in x and in w; Eq. 1): with dLdy given,
 *   dLdx = M^T dLdy                                  (B*C*H*W, must not alias x or dLdy)
 *   dLdw[o][i][a][b] = sum over batch and pixels of dLdy[n][o][r][c] * x[n][i][r-(k-1)+a][c-(k-1)+b]
 *                                                    (C*C*k*k, masked entries 0, deterministic two-pass sum)
 * workspace: device scratch of invconv_bwd_workspace_bytes(B, C, H, W, k) bytes, contents undefined on return.
 */
invconv_status invconv_conv_bwd(const float *x, const float *w, const float *dLdy, float *dLdx, float *dLdw,
                                int B, int C, int H, int W, int k,
                                void *workspace, size_t workspace_bytes, void *stream);

/*
 * Backward pass (Section 3.1-3.3, Eq. 2 and Eq. 4, Theorems 1 and 2).
 *   dLdy = M^{-T} dLdx, M being the matrix of conv_w: the transposed system is
 *          solved by back-substitution over anti-diagonals in decreasing order.
 *   dLdw[o][i][a][b] = - sum_{n,r,c} dLdy[n][o][r][c] * x[n][i][r-(k-1)+a][c-(k-1)+b],
 *          summed over batch and pixels, 0 at masked entries; computed with a
 *          fixed-order two-pass reduction (bitwise reproducible, no atomics).
 *   x [in] output of invconv_fwd    dLdx [in]    dLdy [out] must not alias x or dLdx
 *   dLdw [out] C*C*k*k floats, overwritten (not accumulated)
 *   workspace [scratch] device memory of at least invconv_bwd_workspace_bytes() bytes,
 *          256-byte aligned; contents undefined afterwards.
 */
invconv_status invconv_bwd(const float *x, const float *w, const float *dLdx,
                           float *dLdy, float *dLdw,
                           int B, int C, int H, int W, int k,
                           void *workspace, size_t workspace_bytes, void *stream);

/* Bytes of scratch invconv_bwd needs for this shape; 0 if the shape is invalid or unsupported. */
size_t invconv_bwd_workspace_bytes(int B, int C, int H, int W, int k);

/*
 * invconv_bwd for callers that cannot allocate device memory and have no workspace to pass: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same results;
 * the scratch is an array of INVCONV_STATIC_SCRATCH_BYTES bytes that the library holds in the memory of
 * every device it is loaded on until the process ends.  The call allocates and frees nothing.
 *   - Shapes whose invconv_bwd_workspace_bytes() exceeds INVCONV_STATIC_SCRATCH_BYTES are refused with
 *     INVCONV_ERR_WORKSPACE before anything is launched.
 *   - All calls on one device share that device's array: calls that overlap in time on one device (two
 *     streams, two threads) RACE on it and give undefined dLdw.  Calls that follow each other on one
 *     stream are fine: nothing is expected to survive from one call to the next.
 *   - The array's header (its error word) starts as 0 and is only ever set, as for any workspace.
 */
#define INVCONV_STATIC_SCRATCH_BYTES (8u << 20)
invconv_status invconv_bwd_static(const float *x, const float *w, const float *dLdx,
                                  float *dLdy, float *dLdw,
                                  int B, int C, int H, int W, int k, void *stream);

/*
 * log |det dx/dy| of the inverse convolution for ONE H x W image (Section 4):
 * the Jacobian is triangular, so this is -H*W*sum_c log|w[c][c][k-1][k-1]|,
 * exactly 0 for the paper's unit diagonal.  Independent of the data and of B.
 *   out [out] one device float.
 */
invconv_status invconv_logdet(const float *w, int C, int H, int W, int k,
                              float *out, void *stream);

/*
 * One flow step around the inverse convolution (Section 4.1: an Inv-Conv layer, an Actnorm layer - a
 * per-channel affine map with scale s and bias b - and a 1 x 1 convolution Q, in this order):
 *     x = invconv_w(y),   a[c] = s[c] x[c] + b[c],   z[o] = sum_i Q[o][i] a[i]   at every pixel.
 * Only z is written: for few-channel images that fit on chip (C <= 4, H <= 64, W a multiple of 4, k = 3, or
 * C = 3 with k = 5) and batches of 4 MB or more the three layers run as ONE kernel that reads y and writes z,
 * i.e. the HBM traffic of the inverse convolution alone; for a few such images the kernel that solves one image
 * on several waves applies the two neighbours on its way out (one launch, no set-up launch; the backward pass
 * of k = 3 likewise, plus one small launch that finishes the parameter gradients), and so does the forward pass
 * of 5-16 channels on images of at most 16 rows; other shapes run the same arithmetic as separate passes over
 * scratch.
 *   s, b [in] C floats each;  Q [in] C*C floats, row = output channel; must be invertible (a singular Q
 *   yields inf/NaN like a zero diagonal of w).
 *   z [out] B*C*H*W, must not alias an input.
 *   logdet [out, may be NULL] one device float: log|det dz/dy| of one image (Section 4)
 *       = -H W sum_c log|w[c][c][k-1][k-1]| + H W sum_c log|s[c]| + H W log|det Q|.
 *   workspace: at least invconv_flowstep_workspace_bytes() bytes (the same buffer serves both calls).
 */
invconv_status invconv_flowstep_fwd(const float *y, const float *w, const float *s, const float *b, const float *Q,
                                    float *z, float *logdet, int B, int C, int H, int W, int k,
                                    void *workspace, size_t workspace_bytes, void *stream);

/*
 * Backward pass of that step from its OUTPUT z (x is recomputed on chip as diag(1/s) (Q^-1 z - b), so the
 * forward pass need not keep it).  Chain rule through the three layers (Eq. 2 and Eq. 4 with Theorems 1 and 2
 * for the inverse convolution; the neighbours are linear maps per pixel):
 *   dLdy  = M^-T ( s * Q^T dLdz )                                    B*C*H*W
 *   dLdw  as invconv_bwd, with dL/dx = s * Q^T dLdz                  C*C*k*k, masked entries 0
 *   dLdQ[o][i] = sum dLdz[o] a[i],  dLds[c] = sum (Q^T dLdz)[c] x[c],  dLdb[c] = sum (Q^T dLdz)[c]
 *                                                                    sums over batch and pixels, fixed order
 * plus logdet_weight times the gradient of the step's log-determinant (closed forms, Section 4):
 *   dLdw[c][c][k-1][k-1] -= logdet_weight H W / w[c][c][k-1][k-1],  dLds[c] += logdet_weight H W / s[c],
 *   dLdQ += logdet_weight H W Q^-T.   (A loss that contains `weight * logdet` of one image passes that weight;
 *   0 leaves the data term alone.)
 */
invconv_status invconv_flowstep_bwd(const float *z, const float *w, const float *s, const float *b, const float *Q,
                                    const float *dLdz, float *dLdy, float *dLdw, float *dLds, float *dLdb,
                                    float *dLdQ, float logdet_weight, int B, int C, int H, int W, int k,
                                    void *workspace, size_t workspace_bytes, void *stream);
size_t invconv_flowstep_workspace_bytes(int B, int C, int H, int W, int k);   /* 0 if invalid or unsupported */

/* The same two calls with the form chosen by the caller (for measurement): INVCONV_FLOW_SEPARATE runs the
 * three layers as separate passes over scratch whatever the shape, INVCONV_FLOW_FUSED the fused kernels
 * wherever they exist (separate passes elsewhere); INVCONV_FLOW_AUTO fuses where the fused kernels exist and
 * the batch is large enough for the saved HBM passes to matter. */
enum { INVCONV_FLOW_AUTO = 0, INVCONV_FLOW_SEPARATE = 1, INVCONV_FLOW_FUSED = 2 };
invconv_status invconv_flowstep_fwd_ex(const float *y, const float *w, const float *s, const float *b, const float *Q,
                                       float *z, float *logdet, int B, int C, int H, int W, int k,
                                       void *workspace, size_t workspace_bytes, void *stream, int form);
invconv_status invconv_flowstep_bwd_ex(const float *z, const float *w, const float *s, const float *b, const float *Q,
                                       const float *dLdz, float *dLdy, float *dLdw, float *dLds, float *dLdb,
                                       float *dLdQ, float logdet_weight, int B, int C, int H, int W, int k,
                                       void *workspace, size_t workspace_bytes, void *stream, int form);

/*
 * bf16-STORAGE VARIANT of invconv_fwd / invconv_bwd: the activations (y, x, dLdx, dLdy) are bf16 in memory
 * (16-bit words holding the upper half of an IEEE float, round to nearest even on the way out), the kernel w and
 * its gradient dLdw stay fp32, and all arithmetic is fp32 as in the plain calls.  Half the HBM bytes of the
 * fp32 calls; what matters where a batch is large enough to be bandwidth-bound.  Few-channel images that fit on
 * chip (C <= 4, H <= 64) convert on the way into and out of the on-chip tile; other shapes run the fp32 kernels
 * between conversion passes over scratch.  Results carry bf16's rounding: x and dLdy agree with the fp32 calls
 * on the same (bf16-exact) inputs to 2^-8 relative per element; dLdw is formed from the unrounded dLdy.
 *   y, x, dLdx, dLdy: B*C*H*W 16-bit words (8-byte aligned for the on-chip form).
 *   workspace: at least invconv_bf16_workspace_bytes() bytes.
 */
invconv_status invconv_fwd_bf16(const void *y, const float *w, void *x, int B, int C, int H, int W, int k,
                                void *workspace, size_t workspace_bytes, void *stream);
invconv_status invconv_bwd_bf16(const void *x, const float *w, const void *dLdx, void *dLdy, float *dLdw,
                                int B, int C, int H, int W, int k,
                                void *workspace, size_t workspace_bytes, void *stream);
size_t invconv_bf16_workspace_bytes(int B, int C, int H, int W, int k);   /* 0 if invalid or unsupported */

/* Same operations with an explicit kernel variant (INVCONV_VARIANT_*). */
invconv_status invconv_fwd_ex(const float *y, const float *w, float *x,
                              int B, int C, int H, int W, int k, void *stream, int variant);
invconv_status invconv_bwd_ex(const float *x, const float *w, const float *dLdx,
                              float *dLdy, float *dLdw,
                              int B, int C, int H, int W, int k,
                              void *workspace, size_t workspace_bytes, void *stream, int variant);

/*
 * A stack of L inverse-convolution layers (Section 4.1 repeats the flow step K times), layer l with
 * its own kernel w[l]:  x[0] = invconv(y; w[0]),  x[l] = invconv(x[l-1]; w[l]).
 * `w` and `x` are HOST arrays of L device pointers (read during the call only); every x[l] is a
 * distinct B*C*H*W buffer (all are kept: the backward pass needs them).  Results are those of L
 * calls of invconv_fwd; where the shape allows it the layers run as one pipelined launch in which
 * layer l+1 trails layer l by a few dozen anti-diagonals.  L in 1..16.
 *   workspace: at least invconv_chain_workspace_bytes() bytes of device memory, 256-byte aligned.
 * A stack that needs more workgroups than the device holds at once goes out as several launches of
 * whole layers, so that no workgroup ever waits for one that has not started.
 */
invconv_status invconv_chain_fwd(const float *y, const float *const *w, float *const *x, int L,
                                 int B, int C, int H, int W, int k,
                                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * Backward pass through the same stack: given x[l] (outputs of invconv_chain_fwd), the kernels and
 * dLdx_last = dL/dx[L-1], writes dLdy_first = dL/d(y of layer 0) and dLdw[l] for every layer
 * (Eq. 2 and Eq. 4 per layer; the input gradient of layer l is the output gradient of layer l-1).
 * `x`, `w`, `dLdw` are HOST arrays of L device pointers.  Intermediate gradients live in the workspace.
 */
invconv_status invconv_chain_bwd(const float *const *x, const float *const *w, const float *dLdx_last,
                                 float *dLdy_first, float *const *dLdw, int L,
                                 int B, int C, int H, int W, int k,
                                 void *workspace, size_t workspace_bytes, void *stream);

/* invconv_logdet for every layer of a stack in one launch: out[l] = log|det| of layer l (L device floats). */
invconv_status invconv_chain_logdet(const float *const *w, int L, int C, int H, int W, int k,
                                    float *out, void *stream);

/* Bytes of scratch the two chain calls need (0 if the shape is invalid or unsupported). */
size_t invconv_chain_workspace_bytes(int L, int B, int C, int H, int W, int k);

/* Static, human-readable name of a status code. */
const char *invconv_status_string(invconv_status status);

/* Library version, major*10000 + minor*100 + patch. */
int invconv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* INVCONV_H */
