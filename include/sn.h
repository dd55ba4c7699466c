/*
 * sn.h -- C ABI of the MI355X (gfx950) kernels for the memory-budgeted CNN
 * training step of SuperNeurons (arXiv 1801.04380).
 *
 * The paper's runtime owns all GPU memory; each CONV step is handed whatever
 * bytes are free at that step as "convolution workspace", tries only the
 * algorithms whose workspace fits, and takes the fastest of them (Sec. 3.5).
 * The workspace never changes the result (Sec. 3.5).  The cheap layers (ACT,
 * BN, POOL) are the ones its cost-aware recomputation replays (Sec. 3.4).
 * This library is that layer level: CONV forward / backward-data /
 * backward-filter with an explicit workspace budget, the planner, and the cheap
 * layers, forward and backward.
 *
 * Conventions for every entry point
 *  - All tensor pointers are DEVICE pointers owned by the caller, 16-byte
 *    aligned (workspace: 256-byte aligned).  Shape structs and the size_t /
 *    enum outputs of the query and planner calls are HOST memory.
 *  - The library never allocates, frees or keeps device memory and holds no
 *    pointer after a call returns.  (Its one buffer is the fixed-size array of
 *    sn_conv2d_fwd_noalloc, part of the loaded code object.)
 *  - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *    default stream).  No call synchronises the device.  Outputs are valid once
 *    the stream reaches that point; workspace contents are undefined afterwards.
 *  - Outputs are overwritten, never accumulated into.
 *  - Layouts: activations NCHW, filters KCRS, both dense row-major.
 *    P = floor((H + 2*pad_h - R)/stride_h) + 1, Q likewise.  groups = 1,
 *    dilation = 1, no bias.  The filter is applied as cross-correlation.
 *  - Errors are return codes.  With SN_ERR_BAD_ARG, SN_ERR_UNSUPPORTED and
 *    SN_ERR_WORKSPACE_TOO_SMALL nothing has been launched; SN_ERR_LAUNCH may come after part
 *    of a call's kernels has been enqueued (outputs and workspace are then undefined).
 *  - bf16 values are the upper 16 bits of an IEEE fp32, stored as uint16;
 *    fp32 results are rounded to bf16 to nearest, ties to even.
 */
#ifndef SN_H
#define SN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SN_OK = 0,
    SN_ERR_BAD_ARG = 1,             /* null pointer, misaligned pointer, bad dimension */
    SN_ERR_UNSUPPORTED = 2,         /* valid request this build has no kernel for */
    SN_ERR_WORKSPACE_TOO_SMALL = 3, /* named algorithm needs more workspace than given */
    SN_ERR_LAUNCH = 4               /* the HIP runtime refused a launch */
} sn_status;

typedef enum { SN_F32 = 0, SN_BF16 = 1 } sn_dtype;

typedef enum { SN_CONV_FWD = 0, SN_CONV_BWD_DATA = 1, SN_CONV_BWD_FILTER = 2 } sn_conv_dir;

/* The algorithm menu the planner chooses from (Sec. 3.5: several algorithms,
 * some of which need workspace to reach their speed).
 *  DIRECT       implicit GEMM straight from the NCHW/KCRS tensors; 0 bytes.
 *               Inputs with very few channels (bf16, C * R * S <= 32, W even: a
 *               network's first layer) run a kernel of their own here that
 *               holds the whole reduction in one MFMA operand and is bound by
 *               writing y (forward) or reading dy (backward-filter, also under
 *               STAGED, where its workgroups' partial sums are reduced in a fixed order).
 *               1x1 / stride-1 / unpadded layers (bf16, C and K multiples of 8) run
 *               forward and backward-data as a matrix product per image that
 *               needs no re-laid-out operand, under DIRECT and STAGED alike;
 *               so does backward-data of 1x1 / stride-2 layers on planes of even
 *               size, whose kernel writes each 2x2 cell of dx (one value, three
 *               zeros) itself: sn_conv_workspace_query reports STAGED there with
 *               0 bytes and sn_conv_plan names DIRECT.  Every other strided
 *               backward-data works by residue classes of the input pixels
 *               (h mod stride_h, w mod stride_w): a class shares its taps, so only
 *               the taps that meet an output pixel are multiplied.
 *  IM2COL_GEMM  explicit: unfold patches into a column buffer in the workspace
 *               (as many images per pass as fit), then a GEMM over it; the
 *               backward-data form folds the column gradient back (col2im).
 *  STAGED       implicit GEMM that stages a re-laid-out operand in the
 *               workspace: the filter packed tap-major for forward and
 *               backward-data; per-slice partial sums of dw (reduced in a fixed
 *               order, so the result is run-to-run identical) for
 *               backward-filter (3x3, 1x1, 5x5, 1x7 and 7x1 "same" layers take from a
 *               quarter of the slices they want, min_bytes, up to all of them,
 *               preferred_bytes: fewer slices are fewer, longer workgroups).  On strided shapes (bf16; 1x1 filters without
 *               padding, and filters whose taps reach at most one row / column
 *               of the stride grid beyond the output's, e.g. 3x3 stride 2 pad 1, or
 *               at most two on one side without padding, e.g. 11x11 stride 4)
 *               also the phase planes of the input: x[i*stride + a] for each
 *               residue a becomes a channel group, over which the convolution
 *               has stride 1 and runs on the stride-1 kernels (inner filter
 *               1x1, 2x2 or 3x3 by the span of the tap offsets).  Forward with C a
 *               multiple of 16 and K of 8 needs the planes only as its preferred
 *               workspace for 1x1 filters with 512 output channels or more: below
 *               that, and for every other filter, it gathers the input pixel by
 *               pixel under each tap and stages only the filter with the channel
 *               innermost (min_bytes = K*C*R*S*2; 0 for 1x1 filters, which are that
 *               form already, so DIRECT runs the same kernel).  Otherwise forward and
 *               backward-data take the planes of as many images per pass as the
 *               workspace holds (min_bytes: one image).
 *  WINOGRAD     F(2x2, 3x3) for the fp32 path (3x3 filters, stride 1, forward and
 *               backward-data): the transformed filter, the transformed input
 *               tiles and the 16 products per tile live in the workspace, for as
 *               many images per pass as fit; 2.25 times fewer multiplications.
 *               Sums in a different order than the direct form (fp32 rounding).
 *  AUTO         let the planner pick the fastest algorithm that fits. */
typedef enum {
    SN_ALGO_AUTO = -1,
    SN_ALGO_DIRECT = 0,
    SN_ALGO_IM2COL_GEMM = 1,
    SN_ALGO_STAGED = 2,
    SN_ALGO_WINOGRAD = 3,
    SN_ALGO_COUNT = 4
} sn_conv_algo;

typedef struct {
    int32_t N, C, H, W;        /* input x[N][C][H][W] */
    int32_t K, R, S;           /* filter w[K][C][R][S] */
    int32_t stride_h, stride_w;
    int32_t pad_h, pad_w;
    int32_t in_dtype;          /* sn_dtype of x, w, dy */
    int32_t out_dtype;         /* sn_dtype of y, dx; dw is always fp32.  fp32 in => fp32 out */
} sn_conv_shape;

typedef void *sn_stream;

/* Library version, for the binding's sanity check. */
int sn_version(void);

/* Output size rule used by every CONV and POOL entry point (floor rule; it
 * reproduces the AlexNet tensor sizes of Sec. 4.1).  Returns 0 if the window
 * does not fit. */
int sn_out_dim(int in, int pad, int window, int stride);

/* Workspace needs of one algorithm for one CONV step (Sec. 3.5: an algorithm is
 * memory-feasible iff its workspace fits the free bytes).
 *  min_bytes        least workspace with which the algorithm runs at all
 *  preferred_bytes  workspace beyond which it gets no faster
 * Returns SN_ERR_UNSUPPORTED if the algorithm cannot run this shape. */
sn_status sn_conv_workspace_query(const sn_conv_shape *shape, sn_conv_dir dir, sn_conv_algo algo,
                                  size_t *min_bytes, size_t *preferred_bytes);

/* Planner (Sec. 3.5): among the algorithms whose min_bytes <= budget_bytes pick
 * the fastest.  "Fastest" comes from times recorded for this exact shape by
 * sn_planner_record / sn_conv_autotune (the paper benchmarks the feasible
 * algorithms at run time); a recorded time applies to budgets >= the workspace
 * it was measured with.  With no feasible record the choice falls back to a
 * built-in ranking (WINOGRAD where it applies, C * K >= 8192 and at least 2048 tiles fit a pass, STAGED,
 * then DIRECT; DIRECT first for forward on few-channel inputs).  Among records within 3 % of the fastest the one with the
 * smallest workspace wins (then the faster).  DIRECT needs 0 bytes, so a plan always exists.  bytes_used = the workspace the choice will use
 * (<= budget_bytes).  predicted_ms may be NULL; it receives the recorded time
 * or a negative value if the choice came from the built-in ranking. */
sn_status sn_conv_plan(const sn_conv_shape *shape, sn_conv_dir dir, size_t budget_bytes,
                       sn_conv_algo *algo, size_t *bytes_used, float *predicted_ms);

/* Record / forget measured times (host-side table, process-wide, thread-safe). */
sn_status sn_planner_record(const sn_conv_shape *shape, sn_conv_dir dir, sn_conv_algo algo,
                            size_t workspace_bytes, float ms);
void sn_planner_clear(void);

/* Benchmark every algorithm that fits workspace_bytes on the caller's own
 * buffers (same arguments as the matching sn_conv2d_* call: a, b are its two
 * inputs, out its output) and record the times: per algorithm one untimed launch, then
 * `iters` launches timed one by one, of which the median counts.  Synchronises the stream. */
sn_status sn_conv_autotune(sn_conv_dir dir, const void *a, const void *b, void *out,
                           const sn_conv_shape *shape, void *workspace, size_t workspace_bytes,
                           int iters, sn_stream stream);

/* CONV forward:  y[n,k,p,q] = sum_{c,r,s} x[n,c,p*sh+r-ph,q*sw+s-pw] * w[k,c,r,s]
 * (out-of-image taps contribute 0).  x, w of in_dtype; y of out_dtype.
 * algo = AUTO plans with workspace_bytes as the budget.  A named algorithm whose
 * min_bytes exceeds workspace_bytes returns SN_ERR_WORKSPACE_TOO_SMALL.
 * workspace may be NULL iff workspace_bytes == 0. */
sn_status sn_conv2d_fwd(const void *x, const void *w, void *y, const sn_conv_shape *shape,
                        sn_conv_algo algo, void *workspace, size_t workspace_bytes, sn_stream stream);

/* sn_conv2d_fwd for callers that cannot allocate or pass device memory beyond the tensors
 * themselves: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * It is sn_conv2d_fwd with algo = SN_ALGO_STAGED (same kernels, bit-identical y) whose workspace,
 * the re-laid-out filter, is a fixed array of SN_NOALLOC_SCRATCH_BYTES that the library's code
 * object holds on every GPU it is loaded on until the process ends.  No hipMalloc / hipFree or
 * other allocating call is made.  The first call on a device looks up the array's address there
 * (make that call outside a graph capture).
 *  - SN_ERR_UNSUPPORTED if STAGED has no kernel for the shape (see sn_conv_workspace_query);
 *    SN_ERR_WORKSPACE_TOO_SMALL if its min_bytes exceed SN_NOALLOC_SCRATCH_BYTES (filters of
 *    more than about 4 M elements); nothing is launched then.
 *  - Every call on a GPU uses that GPU's one array: calls that overlap on a GPU (different
 *    streams, or host threads without ordering) race on it; calls on one stream are safe.  The
 *    array keeps the last call's packed filter; each call rewrites all of what it reads. */
#define SN_NOALLOC_SCRATCH_BYTES (8u << 20)
sn_status sn_conv2d_fwd_noalloc(const void *x, const void *w, void *y, const sn_conv_shape *shape,
                                sn_stream stream);

/* CONV forward that also takes, for the BN layer that follows it, the batch statistics of its own
 * output (Sec. 3.4: CONV -> BN -> ReLU is the chain the runtime schedules as a unit): y exactly
 * as sn_conv2d_fwd writes it for the same algo and workspace, and
 *   save_mean[k] = mean over (n,p,q) of y[n,k,p,q], save_invstd[k] = 1/sqrt(biased var + eps),
 * of the values as stored (after rounding to out_dtype), i.e. what sn_bn_fwd(y) would save, up to
 * the order of the sums.  Where a tile kernel runs the CONV (stride 1, bf16 inputs) the
 * statistics come out of its accumulators -- per tile and channel a count, a mean and a sum of
 * squared deviations, combined pairwise in fp64 in a fixed order -- and y is not read again;
 * elsewhere a pass over y follows the CONV.  sn_bn_apply / sn_bn_relu_pool2_apply then finish the
 * BN in one pass.  scratch: device memory of at least sn_conv_bn_stats_scratch_bytes(shape)
 * bytes, 16-byte aligned, contents undefined afterwards (SN_ERR_WORKSPACE_TOO_SMALL if smaller). */
size_t sn_conv_bn_stats_scratch_bytes(const sn_conv_shape *shape);
sn_status sn_conv2d_fwd_bn_stats(const void *x, const void *w, void *y, const sn_conv_shape *shape,
                                 sn_conv_algo algo, void *workspace, size_t workspace_bytes,
                                 float *save_mean, float *save_invstd, float eps,
                                 void *scratch, size_t scratch_bytes, sn_stream stream);

/* CONV backward-data: dx[n,c,h,v] = sum over (k,p,q,r,s) with p*sh+r-ph = h and
 * q*sw+s-pw = v of dy[n,k,p,q] * w[k,c,r,s].  dy, w of in_dtype; dx of out_dtype. */
sn_status sn_conv2d_bwd_data(const void *dy, const void *w, void *dx, const sn_conv_shape *shape,
                             sn_conv_algo algo, void *workspace, size_t workspace_bytes, sn_stream stream);

/* CONV backward-filter: dw[k,c,r,s] = sum_{n,p,q} dy[n,k,p,q] * x[n,c,p*sh+r-ph,q*sw+s-pw].
 * x, dy of in_dtype; dw always fp32.  DIRECT may split the (n,p,q) sum across
 * workgroups and combine with floating-point atomics (sum order not fixed);
 * STAGED and IM2COL_GEMM sum in a fixed order. */
sn_status sn_conv2d_bwd_filter(const void *x, const void *dy, void *dw, const sn_conv_shape *shape,
                               sn_conv_algo algo, void *workspace, size_t workspace_bytes, sn_stream stream);

/* ACT (ReLU), one of the cheap layers recomputation replays (Sec. 3.4):
 * y = x > 0 ? x : 0.  n elements of `dtype`.  y may alias x. */
sn_status sn_relu_fwd(const void *x, void *y, size_t n, sn_dtype dtype, sn_stream stream);

/* dx = x > 0 ? dy : 0.  x may be the layer's input or its output (same gate).
 * dx may alias dy. */
sn_status sn_relu_bwd(const void *x, const void *dy, void *dx, size_t n, sn_dtype dtype, sn_stream stream);

/* BN forward, training mode (Sec. 3.4 cheap layer): per channel c over M = N*H*W,
 *   mean = sum(x)/M, var = sum((x-mean)^2)/M, invstd = 1/sqrt(var+eps),
 *   y = gamma*(x-mean)*invstd + beta.
 * x, y of `dtype` [N][C][H][W]; gamma, beta, save_mean, save_invstd fp32 [C];
 * arithmetic in fp32.  Running statistics are NOT touched, so a replay of this
 * call is side-effect free and gives bit-identical outputs.  y must not alias x
 * (y doubles as scratch for the per-slice partial statistics). */
sn_status sn_bn_fwd(const void *x, const float *gamma, const float *beta, void *y,
                    float *save_mean, float *save_invstd,
                    int N, int C, int H, int W, float eps, sn_dtype dtype, sn_stream stream);

/* BN forward followed by ReLU in one pass, the segment that recomputation replays after a
 * CONV (Sec. 3.4: the cheap layers between two checkpoints are recomputed together):
 *   y = max(gamma*(x-mean)*invstd + beta, 0)   (0 unless the BN output is > 0),
 * everything else as sn_bn_fwd.  The BN output itself is not stored: sn_relu_bwd gates on y,
 * sn_bn_bwd needs x and the saved statistics only, and sn_bn_relu_bwd does both from x. */
sn_status sn_bn_relu_fwd(const void *x, const float *gamma, const float *beta, void *y,
                         float *save_mean, float *save_invstd,
                         int N, int C, int H, int W, float eps, sn_dtype dtype, sn_stream stream);

/* BN forward (optionally with the ReLU, relu != 0) from statistics the caller already has --
 * sn_conv2d_fwd_bn_stats leaves them, or an earlier sn_bn_fwd on the same x: the normalisation
 * pass alone, one read of x and one write of y, with the arithmetic of sn_bn_fwd /
 * sn_bn_relu_fwd (bit-identical y for the same mean and invstd).  y must not alias x. */
sn_status sn_bn_apply(const void *x, const float *gamma, const float *beta,
                      const float *mean, const float *invstd, void *y,
                      int N, int C, int H, int W, int relu, sn_dtype dtype, sn_stream stream);

/* BN backward from the saved statistics, xhat = (x-mean)*invstd:
 *   dbeta = sum(dy), dgamma = sum(dy*xhat),
 *   dx = gamma*invstd/M * (M*dy - dbeta - xhat*dgamma).
 * dx must alias neither x nor dy. */
sn_status sn_bn_bwd(const void *x, const void *dy, const float *gamma,
                    const float *save_mean, const float *save_invstd,
                    void *dx, float *dgamma, float *dbeta,
                    int N, int C, int H, int W, sn_dtype dtype, sn_stream stream);

/* Backward of the BN + ReLU pair (sn_bn_relu_fwd) in one call: sn_bn_bwd applied to
 *   g = y > 0 ? dy : 0,
 * where y is the pair's output as sn_bn_relu_fwd stored it (the ReLU gate of sn_relu_bwd) and
 * dy the gradient that reaches it; g is never stored.  y is not an argument: whether it is
 * > 0 is re-derived from x, gamma, beta and the saved statistics with the forward pass's own
 * arithmetic (including the rounding of the stored value to `dtype`), so the result is
 * bit-identical to gating on the stored y while the pair's output need not be alive, or
 * recomputed (Sec. 3.4), for this call.  gamma, beta, save_mean, save_invstd must be the
 * values the forward call used and wrote.  x is the BN input.  dx must alias neither x nor dy. */
sn_status sn_bn_relu_bwd(const void *x, const void *dy, const float *gamma, const float *beta,
                         const float *save_mean, const float *save_invstd,
                         void *dx, float *dgamma, float *dbeta,
                         int N, int C, int H, int W, sn_dtype dtype, sn_stream stream);

/* BN + ReLU + 2x2 / stride-2 max-pool without padding in one call: the whole run of cheap layers
 * that follows the last CONV of a VGG-style block, which recomputation replays together
 * (Sec. 3.4).  save_mean / save_invstd as sn_bn_fwd; pooled [N][C][H/2][W/2] of `dtype` and idx
 * (int32, same shape) are bit-identical to sn_maxpool_fwd applied to sn_bn_relu_fwd's output,
 * which is not written: nothing after this call needs it (sn_bn_relu_pool2_bwd takes x, the next
 * CONV takes pooled).  H and W must be even and W a multiple of 4 elements (bf16) or 2 (fp32),
 * else SN_ERR_UNSUPPORTED: make the separate calls then.  idx doubles as scratch for the partial
 * statistics; x, pooled and idx must not alias. */
sn_status sn_bn_relu_pool2_fwd(const void *x, const float *gamma, const float *beta, void *pooled, int32_t *idx,
                               float *save_mean, float *save_invstd,
                               int N, int C, int H, int W, float eps, sn_dtype dtype, sn_stream stream);

/* sn_bn_relu_pool2_fwd from statistics the caller already has (as sn_bn_apply): pooled and idx
 * bit-identical to sn_bn_relu_pool2_fwd's for the same mean and invstd.  Same shape limits. */
sn_status sn_bn_relu_pool2_apply(const void *x, const float *gamma, const float *beta,
                                 const float *mean, const float *invstd, void *pooled, int32_t *idx,
                                 int N, int C, int H, int W, sn_dtype dtype, sn_stream stream);

/* Backward of sn_bn_relu_pool2_fwd: sn_bn_relu_bwd applied to the gradient sn_maxpool_bwd would
 * give for (dpooled, idx) -- dpooled of a window goes to the window's winner, 0 elsewhere --
 * formed on the fly, never stored; results bit-identical to the two calls.  Same shape limits;
 * dx [N][C][H][W] must alias none of x, dpooled, idx. */
sn_status sn_bn_relu_pool2_bwd(const void *x, const void *dpooled, const int32_t *idx,
                               const float *gamma, const float *beta,
                               const float *save_mean, const float *save_invstd,
                               void *dx, float *dgamma, float *dbeta,
                               int N, int C, int H, int W, sn_dtype dtype, sn_stream stream);

/* LRN across channels, one of the cheap layers that recomputation replays (Sec. 3.4) and the
 * LRN1 / LRN2 layers of the AlexNet example (Sec. 4).  The paper prints no formula; this is the
 * AlexNet normalisation with alpha divided by the window size (the convention of the library call
 * the paper's runtime makes):
 *   s[n,c,h,w] = k + (alpha / size) * sum over j in [c - size/2, c + size/2], 0 <= j < C, of x[n,j,h,w]^2,
 *   y = x * s^(-beta).
 * size odd, at most 9 (SN_ERR_UNSUPPORTED beyond); alpha >= 0, k > 0.  x, y of `dtype`
 * [N][C][H][W], arithmetic in fp32.  y must not alias x. */
sn_status sn_lrn_fwd(const void *x, void *y, int N, int C, int H, int W,
                     int size, float alpha, float beta, float k, sn_dtype dtype, sn_stream stream);

/* LRN backward from x and dy alone (s is recomputed, y is not needed):
 *   dx_c = dy_c * s_c^(-beta) - (2 * alpha * beta / size) * x_c * sum over j with |j - c| <= size/2
 *          of dy_j * x_j * s_j^(-beta-1).
 * dx must alias neither x nor dy. */
sn_status sn_lrn_bwd(const void *x, const void *dy, void *dx, int N, int C, int H, int W,
                     int size, float alpha, float beta, float k, sn_dtype dtype, sn_stream stream);

/* ReLU and the LRN after it in one pass (the AlexNet-style chain CONV -> ReLU -> LRN; Sec. 3.4: one tensor
 * less to keep or to replay, the ReLU output is never written):
 *   forward   y = LRN(max(x, 0)) with the LRN of sn_lrn_fwd;
 *   backward  dx = (x > 0) ? g : 0 with g = the dx of sn_lrn_bwd on (max(x, 0), dy),
 * i.e. exactly what sn_relu_fwd + sn_lrn_fwd and sn_lrn_bwd + sn_relu_bwd give, from x (the CONV output) alone.
 * Arguments, layouts and errors as for sn_lrn_fwd / sn_lrn_bwd. */
sn_status sn_relu_lrn_fwd(const void *x, void *y, int N, int C, int H, int W,
                          int size, float alpha, float beta, float k, sn_dtype dtype, sn_stream stream);
sn_status sn_relu_lrn_bwd(const void *x, const void *dy, void *dx, int N, int C, int H, int W,
                          int size, float alpha, float beta, float k, sn_dtype dtype, sn_stream stream);

/* Ceilings of the device for the roofline figures (the fractions the benchmark reports are quoted
 * against the datasheet peaks; these are what this GPU reaches in the plainest possible kernel):
 *  MFMA_BF16 / MFMA_F32  a register-resident loop of 32x32x16 bf16 / 32x32x2 fp32 MFMAs on every
 *                        compute unit -> *value in TFLOP/s;
 *  MFMA_BF16_FED         the bf16 loop with its operands arriving as the 3x3 tile kernels get them
 *                        (a wave of 64 channels x 128 pixels; per 24 MFMAs six 1 KB filter items
 *                        from a 2 MiB L2-resident buffer and six pixel operands from LDS; per 72
 *                        MFMAs 32 bytes per thread from memory into LDS behind a barrier; two
 *                        workgroups per compute unit), trivial addresses, nothing transposed or
 *                        stored: what the operand streams alone leave of the peak -> TFLOP/s;
 *  COPY / READ / WRITE   a streaming kernel, 16 bytes per lane, over buf (COPY: first half to
 *                        second half, read + written bytes counted) -> *value in GB/s.  Give it a
 *                        buffer well beyond the 256 MB memory-side cache.
 * buf: device memory, 256-byte aligned, at least 2 MiB for the MFMA kinds (4 MiB for MFMA_BF16_FED);
 * it is overwritten.
 * The best of `iters` timed launches counts.  Synchronises the stream. */
typedef enum { SN_CEIL_MFMA_BF16 = 0, SN_CEIL_MFMA_F32 = 1, SN_CEIL_COPY = 2, SN_CEIL_READ = 3, SN_CEIL_WRITE = 4,
               SN_CEIL_MFMA_BF16_FED = 5 } sn_ceiling_kind;
sn_status sn_measure_ceiling(sn_ceiling_kind kind, void *buf, size_t buf_bytes, int iters, sn_stream stream,
                             double *value);

/* POOL (max) forward, the paper's example of a cheap-to-recompute layer
 * (Sec. 3.4).  Window kh x kw, stride, padding (pad < window; padded positions
 * never win).  Of equal maxima the first in row-major window order wins.
 * idx[n,c,p,q] = h*W + v of the winner inside its input plane (int32). */
sn_status sn_maxpool_fwd(const void *x, void *y, int32_t *idx, int N, int C, int H, int W,
                         int kh, int kw, int sh, int sw, int ph, int pw,
                         sn_dtype dtype, sn_stream stream);

/* POOL backward: dx[n,c,i] = sum of dy[n,c,p,q] over the windows whose idx is i
 * (overlapping windows add; fp32 accumulation in window order). */
sn_status sn_maxpool_bwd(const void *dy, const int32_t *idx, void *dx, int N, int C, int H, int W,
                         int kh, int kw, int sh, int sw, int ph, int pw,
                         sn_dtype dtype, sn_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* SN_H */
