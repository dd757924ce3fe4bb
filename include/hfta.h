/*
 * hfta.h -- C ABI of the horizontally fused training-array operators for one
 * AMD Instinct MI355X (gfx950).
 *
 * B independent training jobs of one architecture (same operator shapes,
 * different hyper-parameters) are run as ONE fused job: every operator below
 * processes the tensors of all B models in one launch and is, per model,
 * mathematically the ordinary single-model operator (paper section "Our
 * Proposal: HFTA"; appendix "HFTA Operator Fusion Rules", the fusion rules
 * table).  The kernels are hand-written HIP; nothing is delegated to a vendor
 * library.
 *
 * Conventions common to every entry point
 * ---------------------------------------
 *  - Return value: HFTA_OK or a negative hfta_status.  No exceptions, aborts
 *    or prints.  All argument validation happens before any launch, so every
 *    HFTA_EINVAL / HFTA_EUNSUPPORTED / HFTA_EWORKSPACE path works on a host
 *    without a GPU.
 *  - Pointers are DEVICE pointers unless a comment says "host".  The caller
 *    owns all memory; the library allocates nothing, frees nothing and keeps
 *    no pointer after the call returns.  The only state it keeps between calls
 *    is read-only after its first use: the compute-unit count of the device
 *    (queried once, sizes the persistent GEMM launches), for
 *    hfta_linear_fwd_static the address of its built-in scratch array, and a
 *    memo of LDS pitches per convolution geometry (a pure function of the
 *    shape, computed on the host the first time a shape is seen).  Scratch memory is a caller-supplied
 *    `workspace` whose required size the matching *_workspace_bytes function
 *    returns (0 = none needed; then NULL is accepted).
 *  - Calls are asynchronous on `stream` (a hipStream_t passed as void*; NULL =
 *    the default stream).  Outputs must not alias inputs unless stated.
 *  - `dtype` is the storage type of activations, activation gradients and the
 *    weights the GEMMs read: HFTA_F32 or HFTA_BF16.  Accumulation is always
 *    fp32.  Parameter gradients (dW, dbias, dgamma, dbeta), BatchNorm /
 *    LayerNorm statistics, optimiser state and master weights are always fp32.
 *    A tensor stored in bf16 is rounded once, to nearest even, from the fp32
 *    accumulator at the store.
 *  - Strided activations: a tensor with logical index (b, n, c, l) -- model,
 *    sample, channel, position -- is described by four element strides
 *    s[4] = {stride_b, stride_n, stride_c, stride_l} (host array).  The
 *    paper's convolution layout [N, B*C, L] is {C*L, B*C*L, L, 1}; its linear
 *    layout [B, N, F] is {N*F, F, 1, -} with L = 1.
 *  - Per-model hyper-parameters are device arrays of length B (fp32) that the
 *    kernels read themselves (section "Our Proposal: HFTA", paragraph "HFTA
 *    Optimizers and Learning Rate Schedulers").
 *  - Sizes are limited to 2^31-1 elements per model slice where noted.
 */
#ifndef HFTA_H
#define HFTA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum hfta_status {
  HFTA_OK = 0,
  HFTA_EINVAL = -1,       /* null pointer, B <= 0, non-positive size, bad enum, overflow */
  HFTA_EUNSUPPORTED = -2, /* valid but not implemented (dtype / stride / kernel-size combination) */
  HFTA_EWORKSPACE = -3,   /* workspace missing or too small */
  HFTA_ELAUNCH = -4       /* the HIP runtime reported an error at launch */
} hfta_status;

typedef enum hfta_dtype { HFTA_F32 = 0, HFTA_BF16 = 1 } hfta_dtype;

typedef enum hfta_act {
  HFTA_ACT_NONE = 0,
  HFTA_ACT_RELU = 1,  /* max(x, 0); gradient 0 at x <= 0 */
  HFTA_ACT_LEAKY = 2, /* x > 0 ? x : slope*x; gradient `slope` at x <= 0 */
  HFTA_ACT_TANH = 3,
  HFTA_ACT_GELU = 4   /* exact: x * Phi(x), Phi via erf */
} hfta_act;

const char* hfta_status_string(int status);
int hfta_version(void);

/* ------------------------------------------------------------------------
 * Fused Linear (fusion rules table, row "Linear" -> baddbmm).
 *   X:[B][M][Fx]  W:[B][Fx][Fy]  bias:[B][Fy] (or NULL)  Y:[B][M][Fy], all
 *   contiguous, storage `dtype`.  Per model b: Y[b] = act(X[b] W[b] + bias[b]).
 *   `act` is applied to the fp32 accumulator before the single store.
 * ---------------------------------------------------------------------- */
int hfta_linear_fwd(int B, int M, int Fx, int Fy, int dtype,
                    const void* X, const void* W, const void* bias, void* Y,
                    int act, float act_slope, void* stream);

/* The same operation with a workspace.  With few rows per model (M <= 64: a fully connected head
 * fed by one pooled vector per sample) the reduction over Fx is cut into pieces that run on
 * different compute units; fp32 partial products [split][B][M][Fy] pass through the workspace and a
 * second launch adds them in a fixed order, then bias and act.  Results equal hfta_linear_fwd's up
 * to fp32 summation order.  hfta_linear_fwd_workspace_bytes is 0 where no split is used (then the
 * call is hfta_linear_fwd); EWORKSPACE below that size. */
size_t hfta_linear_fwd_workspace_bytes(int B, int M, int Fx, int Fy, int dtype);
int hfta_linear_fwd_ws(int B, int M, int Fx, int Fy, int dtype,
                       const void* X, const void* W, const void* bias, void* Y,
                       int act, float act_slope, void* workspace, size_t ws_bytes, void* stream);

/* hfta_linear_fwd_ws for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the split partials live in a device array
 * of HFTA_LINEAR_FWD_STATIC_BYTES that is part of the library image, so the call takes no workspace
 * and makes no allocation.  Same arguments, results and validation as hfta_linear_fwd_ws (bit-equal:
 * same kernels, same split count).  HFTA_EWORKSPACE when the partials of the shape exceed the array
 * (hfta_linear_fwd_workspace_bytes(...) > hfta_linear_fwd_static_max_bytes()); HFTA_ELAUNCH when the
 * array's address cannot be obtained on the current device.  Every GPU the library runs on holds its
 * own copy of the array until the process ends; its address is looked up once per device (the one
 * piece of state the library keeps).  All calls on one GPU share the array: calls that overlap there
 * (different streams or threads) race; calls on one stream do not.  Nothing in it needs clearing:
 * each call writes every partial it later reads. */
#define HFTA_LINEAR_FWD_STATIC_BYTES (8u << 20)
size_t hfta_linear_fwd_static_max_bytes(void);
int hfta_linear_fwd_static(int B, int M, int Fx, int Fy, int dtype,
                           const void* X, const void* W, const void* bias, void* Y,
                           int act, float act_slope, void* stream);

/* Backward of hfta_linear_fwd with act = NONE (apply hfta_act_bwd first otherwise).
 *   dX[b] = dY[b] W[b]^T   (storage dtype; NULL = skip)
 *   dW[b] = X[b]^T dY[b]   (fp32 [B][Fx][Fy]; NULL = skip)
 *   dbias[b] = column sums of dY[b]  (fp32 [B][Fy]; NULL = skip)
 * Workspace: hfta_linear_bwd_workspace_bytes (split-K partials of dW). */
size_t hfta_linear_bwd_workspace_bytes(int B, int M, int Fx, int Fy, int dtype);
int hfta_linear_bwd(int B, int M, int Fx, int Fy, int dtype,
                    const void* X, const void* W, const void* dY,
                    void* dX, float* dW, float* dbias,
                    void* workspace, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Fused Conv1d with kernel length 1 (row "Conv1d" -> grouped Conv1d, G = B).
 *   X: logical [B][Nb][Ci][L] with strides xs; Y: [B][Nb][Co][L] with strides
 *   ys; both need stride_l == 1.  W:[B][Co][Ci] contiguous (= the paper's
 *   [B*Co, Ci, 1]), bias:[B][Co] or NULL, storage dtype.
 *   Y[b,n,o,l] = act(bias[b,o] + sum_c W[b,o,c] X[b,n,c,l]).
 * ---------------------------------------------------------------------- */
int hfta_conv1x1_fwd(int B, int Nb, int Ci, int Co, int L, int dtype,
                     const void* X, const int64_t xs[4], const void* W, const void* bias,
                     void* Y, const int64_t ys[4], int act, float act_slope, void* stream);

/* The same convolution with a per-(sample, channel) term in place of the per-channel bias (rows
 * "Conv1d" and the element-wise rows; used where the layer's input is a concatenation of per-point
 * feature maps with vectors tiled along the points: the tiled part's product with its block of the
 * weights does not depend on the point, so it is computed once per sample and enters here):
 *   Y[b,n,o,l] = act(S[b,n,o] + sum_c W[b,o,c] X[b,n,c,l]),   S: [b][n][o] with strides ss[3], ss[2] == 1,
 * storage dtype; the sum is formed in the fp32 accumulator and stored once (no separate pass over Y,
 * where hfta_add_sample_bias would re-read and re-round it).  A per-channel bias, if any, is part of S.
 * Other arguments, layouts and errors as hfta_conv1x1_fwd. */
int hfta_conv1x1_fwd_sample_bias(int B, int Nb, int Ci, int Co, int L, int dtype,
                                 const void* X, const int64_t xs[4], const void* W,
                                 const void* S, const int64_t ss[3],
                                 void* Y, const int64_t ys[4], int act, float act_slope, void* stream);

/* Fused Conv1d k=1 followed by training-mode BatchNorm and an activation (the per-point layers of
 * the point-cloud models; rows "Conv1d" and "BatchNorm1d" of the fusion rules table):
 *   Z = W X + bias                        (stored with strides zs: the BatchNorm backward reads it)
 *   Y = act(gamma (Z - mean) invstd + beta), statistics over (n, l) per (b, c) of the STORED Z.
 * Arguments as in hfta_conv1x1_fwd and hfta_bn_fwd; act in {NONE, RELU, LEAKY} applies to Y.
 * Results equal hfta_conv1x1_fwd followed by hfta_bn_fwd up to the fp32 summation order of the
 * statistics.  With a workspace of hfta_conv1x1_bn_fwd_workspace_bytes (8-byte aligned) and a bf16
 * layer that the streaming convolution kernel takes, the convolution's epilogue leaves per-slice
 * sums there and Z is read once (for the normalisation) instead of twice; otherwise the two
 * operators run one after the other (no workspace needed).  Y == NULL: only Z and the statistics
 * are produced (a consumer that normalises Z on load follows, see hfta_conv1x1_bn_prenorm_fwd). */
size_t hfta_conv1x1_bn_fwd_workspace_bytes(int B, int Nb, int Ci, int Co, int L, int dtype);
int hfta_conv1x1_bn_fwd(int B, int Nb, int Ci, int Co, int L, int dtype,
                        const void* X, const int64_t xs[4], const void* W, const void* bias,
                        const float* gamma, const float* beta, float eps, float momentum,
                        float* running_mean, float* running_var, float* save_mean, float* save_invstd,
                        void* Z, const int64_t zs[4], void* Y, const int64_t ys[4],
                        int act, float act_slope, void* workspace, size_t ws_bytes, void* stream);

/* Backward: dX[b,n,c,l] = sum_o W[b,o,c] dY[b,n,o,l]   (storage dtype, strides dxs; NULL = skip)
 *           dW[b,o,c]   = sum_{n,l} dY[b,n,o,l] X[b,n,c,l]   (fp32; NULL = skip)
 *           dbias[b,o]  = sum_{n,l} dY[b,n,o,l]              (fp32; NULL = skip)
 * The reduction over n and l is split across workgroups; partial sums go to
 * the workspace and are added in a fixed order (bit-reproducible).  With a
 * 256-byte aligned workspace of hfta_conv1x1_bwd_workspace_bytes the data
 * gradient of a narrow bf16 layer (Co <= 128) runs as a streaming k=1
 * convolution of dY with W^T, which is written to the workspace first; with
 * a smaller or NULL workspace dX takes the general GEMM path (same result up
 * to fp32 summation order).  EWORKSPACE only if dW is asked for and its
 * partial sums do not fit. */
size_t hfta_conv1x1_bwd_workspace_bytes(int B, int Nb, int Ci, int Co, int L, int dtype);
int hfta_conv1x1_bwd(int B, int Nb, int Ci, int Co, int L, int dtype,
                     const void* X, const int64_t xs[4], const void* W,
                     const void* dY, const int64_t dys[4],
                     void* dX, const int64_t dxs[4], float* dW, float* dbias,
                     void* workspace, size_t ws_bytes, void* stream);

/* Backward of the block hfta_conv1x1_bn_fwd computes (rows "Conv1d" and "BatchNorm1d" of the fusion
 * rules table), BatchNorm backward and convolution backward in one call:
 *   g  = dY * act'(gamma xhat + beta),  xhat = (Z - mean) invstd        (dY: gradient at the block's output Y)
 *   dZ = gamma invstd (g - mean_{n,l}(g) - xhat mean_{n,l}(g xhat)),  rounded to the storage dtype
 *   dgamma[b,c] = sum g xhat,  dbeta[b,c] = sum g                       (fp32)
 *   dX, dW as hfta_conv1x1_bwd with dZ as its dY;  dbias[b,o] = sum_{n,l} dZ   (fp32, NULL = skip)
 * i.e. the results of hfta_bn_bwd followed by hfta_conv1x1_bwd with dZ stored in between, up to the
 * fp32 summation order.  X, Z, dY, dX: logical [B][Nb][C][L] with strides, stride_l == 1; W as in
 * hfta_conv1x1_fwd (may be NULL when dX is NULL); gamma, beta, save_mean, save_invstd: [B][Co] fp32
 * as hfta_bn_fwd left them.  dX == NULL skips the data gradient (a network's first layer); dX must
 * not overlap X, Z or dY (it is written while other slices of those are still being read).
 * bf16 layers with Ci <= 128, Co <= 128, L % 4 == 0, 8-byte aligned X, Z, dY (and dX) and strides
 * that are multiples of 4 elements run as one
 * reduction kernel (dgamma, dbeta and per-channel constants) plus ONE streaming kernel that forms
 * dZ per 128-point slice in registers and feeds it to both products from LDS: dZ never goes to
 * device memory.  The workspace (hfta_conv1x1_bn_bwd_workspace_bytes, 256-byte aligned) then holds
 * the constants and the per-workgroup fp32 partials of dW and dbias, added in a fixed order
 * (bit-reproducible).  Every other shape or dtype runs the two single operators with dZ in the
 * workspace (the query returns that larger size for them).  A shape the streaming kernel takes
 * whose pointers or strides break its alignment rules needs the larger workspace as well:
 * HFTA_EWORKSPACE if it is not there.  Nothing is allocated.
 * hfta_conv1x1_bn_bwd_one_pass returns 1 for the shapes and dtype of the one-kernel form, else 0 (a
 * caller that already owns a dZ-sized buffer may prefer the two single operators for the others).
 * sums (optional, [B][Co][2] fp32): the two reductions {sum g, sum g xhat} of this block, as the
 * backward call of the block that consumed Y left them (in_sums of hfta_conv1x1_bn_prenorm_bwd);
 * the one-kernel form then skips its reduction pass over dY and Z (dgamma, dbeta and dZ come from
 * these sums; equal to the pass's own up to the fp32 summation order).  Other forms ignore it. */
int hfta_conv1x1_bn_bwd_one_pass(int B, int Nb, int Ci, int Co, int L, int dtype);
size_t hfta_conv1x1_bn_bwd_workspace_bytes(int B, int Nb, int Ci, int Co, int L, int dtype);
int hfta_conv1x1_bn_bwd(int B, int Nb, int Ci, int Co, int L, int dtype,
                        const void* X, const int64_t xs[4], const void* W,
                        const void* Z, const int64_t zs[4], const void* dY, const int64_t dys[4],
                        const float* gamma, const float* beta, const float* save_mean, const float* save_invstd,
                        void* dX, const int64_t dxs[4], float* dW, float* dbias, float* dgamma, float* dbeta,
                        const float* sums, int act, float act_slope, void* workspace, size_t ws_bytes, void* stream);

/* The same two calls for a chain of such blocks in which the activated tensor between two blocks is
 * never stored (rows "Conv1d" and "BatchNorm1d"; the per-point layers of the point-cloud models):
 * the input is given as the PREVIOUS block's stored pre-activation Xpre (strides xs) together with
 * that block's BatchNorm constants in_gamma, in_beta, in_mean, in_invstd ([B][Ci] fp32, as
 * hfta_bn_fwd left them) and its activation in_act in {NONE, RELU, LEAKY}; the kernels form
 *   X = in_act(in_gamma (Xpre - in_mean) in_invstd + in_beta),  rounded to the storage dtype,
 * on the way into LDS with the arithmetic of hfta_bn_fwd, i.e. the very values that block would
 * have stored, and proceed as hfta_conv1x1_bn_fwd / hfta_conv1x1_bn_bwd on that X (in the backward
 * call dX is the gradient with respect to X, what the previous block's backward takes as its dY).
 * Results are bit-identical to storing X and calling the plain pair.  The previous block is run
 * with Y == NULL.  Only the shapes both streaming kernels take: bf16, Ci % 8 == 0, Ci <= 128,
 * 64 <= Co <= 128, L % 4 == 0 (hfta_conv1x1_bn_prenorm_supported returns 1), 8-byte aligned
 * tensors with strides that are multiples of 4 elements; anything else is HFTA_EUNSUPPORTED with
 * nothing launched (store the activated tensor and use the plain pair).  Workspaces:
 * hfta_conv1x1_bn_fwd_workspace_bytes and hfta_conv1x1_bn_bwd_workspace_bytes, required here
 * (HFTA_EWORKSPACE).  Y may be NULL in the forward call, dX in the backward call.
 * The backward call can hand the previous block's BatchNorm backward its two reductions: with
 * in_sums ([B][Ci][2] fp32, optional; needs dX) it also leaves, per input channel,
 *   in_sums[b,c] = {sum g, sum g xhat},  g = dX * in_act'(.),  xhat = (Xpre - in_mean) in_invstd,
 * summed over samples and points with dX as stored -- the thread that loads a piece of Xpre is the
 * one that stores that piece of dX, so this costs no memory traffic -- and the previous block's
 * backward call, given them as `sums`, skips its own pass over dX and Xpre.  Built for Ci <= 64
 * (hfta_conv1x1_bn_prenorm_bwd_gives_sums returns 1; otherwise in_sums != NULL is
 * HFTA_EUNSUPPORTED).  sums: as in hfta_conv1x1_bn_bwd. */
int hfta_conv1x1_bn_prenorm_supported(int B, int Nb, int Ci, int Co, int L, int dtype);
int hfta_conv1x1_bn_prenorm_bwd_gives_sums(int B, int Nb, int Ci, int Co, int L, int dtype);
int hfta_conv1x1_bn_prenorm_fwd(int B, int Nb, int Ci, int Co, int L, int dtype,
                                const void* Xpre, const int64_t xs[4],
                                const float* in_gamma, const float* in_beta, const float* in_mean,
                                const float* in_invstd, int in_act, float in_slope,
                                const void* W, const void* bias, const float* gamma, const float* beta,
                                float eps, float momentum, float* running_mean, float* running_var,
                                float* save_mean, float* save_invstd, void* Z, const int64_t zs[4],
                                void* Y, const int64_t ys[4], int act, float act_slope,
                                void* workspace, size_t ws_bytes, void* stream);
int hfta_conv1x1_bn_prenorm_bwd(int B, int Nb, int Ci, int Co, int L, int dtype,
                                const void* Xpre, const int64_t xs[4],
                                const float* in_gamma, const float* in_beta, const float* in_mean,
                                const float* in_invstd, int in_act, float in_slope,
                                const void* W, const void* Z, const int64_t zs[4],
                                const void* dY, const int64_t dys[4],
                                const float* gamma, const float* beta, const float* save_mean, const float* save_invstd,
                                void* dX, const int64_t dxs[4], float* dW, float* dbias, float* dgamma, float* dbeta,
                                const float* sums, float* in_sums,
                                int act, float act_slope, void* workspace, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Fused Conv2d (row "Conv2d" -> grouped Conv2d with G = B; g = 1 per model).
 *   X:[Nb][B*Ci][H][W]  Wt:[B*Co][Ci][kh][kw]  bias:[B*Co] or NULL
 *   Y:[Nb][B*Co][Ho][Wo], Ho = (H + 2 pad - kh)/stride + 1, all contiguous.
 *   Cross-correlation with zero padding, no dilation.
 * The same two entry points serve the fused ConvTranspose2d (row "ConvT2d"):
 *   ConvT fwd  (x:[Nb][B*Cx][H][W], w:[B*Cx][Cy][kh][kw]) = hfta_conv2d_grouped_bwd's dX
 *              with dY := x, Wt := w, Ci := Cy, Co := Cx  (bias added by hfta_bias_act_nchw);
 *   ConvT bwd-data = hfta_conv2d_grouped_fwd; ConvT dW = hfta_conv2d_grouped_bwd's dW with the
 *              roles of X and dY exchanged the same way.
 * ---------------------------------------------------------------------- */
/* Which kernels run (results agree to the storage tolerance, up to fp32 summation order):
 *  - bf16, 4x4 kernel, stride 2, pad 1, output sides powers of two (>= 4): an implicit GEMM with the
 *    samples folded into the GEMM's columns; needs no workspace.  With a 16-byte aligned workspace of
 *    hfta_conv2d_grouped_fwd_workspace_bytes, layers with few output tiles and a long reduction
 *    split the reduction and keep fp32 partial slices there.
 *  - kernel = image and pad 0 (one output pixel): the fused Linear over the flattened window.
 *  - everything else (other kernels / strides, odd grids, fp32): with a 256-byte aligned workspace of
 *    hfta_conv2d_grouped_fwd_workspace_bytes the convolution is lowered through a column buffer onto
 *    the batched GEMM kernels; with NULL / less it runs as an implicit GEMM per (model, sample).
 * The workspace is scratch: nothing in it is read from an earlier call or kept for a later one. */
size_t hfta_conv2d_grouped_fwd_workspace_bytes(int B, int Nb, int Ci, int Co, int H, int W,
                                               int kh, int kw, int stride, int pad, int dtype);
int hfta_conv2d_grouped_fwd(int B, int Nb, int Ci, int Co, int H, int W, int kh, int kw,
                            int stride, int pad, int dtype,
                            const void* X, const void* Wt, const void* bias, void* Y,
                            int act, float act_slope, void* workspace, size_t ws_bytes, void* stream);

/* dX:[Nb][B*Ci][H][W] storage dtype (NULL = skip); dW: fp32 [B*Co][Ci][kh][kw] (NULL = skip);
 * dbias: fp32 [B*Co] (NULL = skip).
 * Workspace (256-byte aligned): hfta_conv2d_grouped_bwd_min_workspace_bytes is what the implicit-GEMM
 * kernels need -- the weight gradient's split partials and, for the bf16 4x4 / stride 2 / pad 1
 * shapes, the data gradient's weights regrouped per output-parity class (rewritten on every call) --
 * and may be 0; with less, the data gradient falls back to a kernel that gathers single taps and a
 * split weight gradient returns HFTA_EWORKSPACE.  hfta_conv2d_grouped_bwd_workspace_bytes (>= the
 * minimum) additionally enables the column-buffer lowering for the shapes that have no
 * sample-folded kernel.  At most 4 input channels (bf16, 4x4 / stride 2 / pad 1): the data gradient
 * is computed by direct vector arithmetic and needs no workspace. */
size_t hfta_conv2d_grouped_bwd_workspace_bytes(int B, int Nb, int Ci, int Co, int H, int W,
                                               int kh, int kw, int stride, int pad, int dtype);
size_t hfta_conv2d_grouped_bwd_min_workspace_bytes(int B, int Nb, int Ci, int Co, int H, int W,
                                                   int kh, int kw, int stride, int pad, int dtype);
int hfta_conv2d_grouped_bwd(int B, int Nb, int Ci, int Co, int H, int W, int kh, int kw,
                            int stride, int pad, int dtype,
                            const void* X, const void* Wt, const void* dY,
                            void* dX, float* dW, float* dbias,
                            void* workspace, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Fused BatchNorm (rows "BatchNorm1d", "BatchNorm2d"): training mode here, evaluation mode in
 * hfta_bn_eval_fwd below.
 *   X, Y: logical [B][Nb][C][L] with strides xs / ys; supported layouts:
 *   stride_l == 1 (conv family; L = H*W for 2d) or L == 1 && stride_c == 1
 *   (the table's [N, B, C] case).  gamma, beta, running_*, save_*: fp32 [B][C].
 *   Per channel (b,c) over (n,l): mu = mean x; var = mean (x-mu)^2 (biased);
 *   y = act(gamma (x-mu)/sqrt(var+eps) + beta);
 *   running_mean <- (1-momentum) running_mean + momentum mu; running_var likewise
 *   with the unbiased variance (skipped when running_mean == NULL).
 *   save_mean / save_invstd receive mu and 1/sqrt(var+eps) for the backward.
 *   Models never share statistics.
 * ---------------------------------------------------------------------- */
int hfta_bn_fwd(int B, int Nb, int C, int L, int dtype,
                const void* X, const int64_t xs[4], const float* gamma, const float* beta,
                float eps, float momentum, float* running_mean, float* running_var,
                float* save_mean, float* save_invstd,
                void* Y, const int64_t ys[4], int act, float act_slope, void* stream);

/* Normalisation with GIVEN statistics (row "BatchNorm1d"): Y = act(gamma (X - mean) invstd + beta) with
 * mean, invstd [B][C] fp32 as hfta_bn_fwd saved them: the second pass of hfta_bn_fwd alone, bit-identical
 * to what it stored.  For a consumer that dropped an activated tensor (hfta_conv1x1_bn_prenorm_fwd) and
 * wants it back, e.g. to recompute or to inspect it.  Conv layouts (stride_l == 1); nothing is updated. */
int hfta_bn_apply_fwd(int B, int Nb, int C, int L, int dtype, const void* X, const int64_t xs[4],
                      const float* gamma, const float* beta, const float* mean, const float* invstd,
                      void* Y, const int64_t ys[4], int act, float act_slope, void* stream);

/* Evaluation mode of the same rows (the fused operator keeps every argument of the single-model one,
 * its training flag included; with the flag off the running estimates replace the batch statistics):
 *   y = act(gamma (x - running_mean) / sqrt(running_var + eps) + beta); nothing is updated or saved.
 * Layouts, dtypes and activations as hfta_bn_fwd; X is read once, Y written once; Y may alias X.
 * EINVAL on null pointers or non-positive sizes; EUNSUPPORTED for other layouts or activations. */
int hfta_bn_eval_fwd(int B, int Nb, int C, int L, int dtype,
                     const void* X, const int64_t xs[4], const float* gamma, const float* beta,
                     const float* running_mean, const float* running_var, float eps,
                     void* Y, const int64_t ys[4], int act, float act_slope, void* stream);

/* Backward of hfta_bn_fwd including its fused activation (ReLU / LeakyReLU / NONE):
 * the activation mask is recomputed from X and the saved statistics in fp32,
 * exactly as the forward computed it.
 *   dY: gradient w.r.t. the activated output; dX: gradient w.r.t. X (storage dtype);
 *   dgamma, dbeta: fp32 [B][C].
 *   dx_sum (fp32 [B][C], NULL = skip): per-channel sum over (n, l) of dX as stored.  When X was
 *   produced by a fused Linear / Conv with a bias, this IS that layer's bias gradient, obtained
 *   without another pass over dX. */
int hfta_bn_bwd(int B, int Nb, int C, int L, int dtype,
                const void* X, const int64_t xs[4], const void* dY, const int64_t dys[4],
                const float* gamma, const float* beta,
                const float* save_mean, const float* save_invstd,
                void* dX, const int64_t dxs[4], float* dgamma, float* dbeta, float* dx_sum,
                int act, float act_slope, void* stream);

/* ------------------------------------------------------------------------
 * Max-pool over the point axis (PointNet's global feature; section
 * "Methodology", PointNet workload).
 *   X: logical [B][Nb][C][L], stride_l == 1.  V: logical [B][Nb][C] with strides
 *   vs[3] = {stride_b, stride_n, stride_c} (so the result can land directly in
 *   the linear layout [B][Nb][C]); idx: int32, same strides as V.
 *   V = max_l X, idx = the LOWEST l attaining it.  NaN inputs: undefined.
 * ---------------------------------------------------------------------- */
int hfta_maxpool_points(int B, int Nb, int C, int L, int dtype,
                        const void* X, const int64_t xs[4],
                        void* V, int32_t* idx, const int64_t vs[3], void* stream);

/* dX[b,n,c,l] = (l == idx[b,n,c]) ? dV[b,n,c] : 0; dX is fully written. */
int hfta_maxpool_points_bwd(int B, int Nb, int C, int L, int dtype,
                            const void* dV, const int32_t* idx, const int64_t vs[3],
                            void* dX, const int64_t dxs[4], void* stream);

/* ------------------------------------------------------------------------
 * BatchNorm + activation + point max-pool as one operator (PointNet's global feature is
 * max_l act(BN(z))).  Same arguments as hfta_bn_fwd / hfta_maxpool_points; the activated
 * tensor is never materialised.  Results are bit-identical to hfta_bn_fwd followed by
 * hfta_maxpool_points: the maximum is taken over the activated values rounded to the storage
 * dtype, lowest index on ties.  X needs stride_l == 1.
 * Backward: dX = BatchNorm backward of the gradient that is dV[b,n,c] at l == idx[b,n,c] and 0
 * elsewhere (equal to hfta_maxpool_points_bwd followed by hfta_bn_bwd up to fp32 summation
 * order); indices outside [0, L) are clamped.  dx_sum as in hfta_bn_bwd.
 * ---------------------------------------------------------------------- */
int hfta_bn_fwd_maxpool(int B, int Nb, int C, int L, int dtype,
                        const void* X, const int64_t xs[4], const float* gamma, const float* beta,
                        float eps, float momentum, float* running_mean, float* running_var,
                        float* save_mean, float* save_invstd,
                        void* V, int32_t* idx, const int64_t vs[3], int act, float act_slope, void* stream);
int hfta_bn_bwd_maxpool(int B, int Nb, int C, int L, int dtype,
                        const void* X, const int64_t xs[4], const void* dV, const int32_t* idx,
                        const int64_t vs[3], const float* gamma, const float* beta,
                        const float* save_mean, const float* save_invstd,
                        void* dX, const int64_t dxs[4], float* dgamma, float* dbeta, float* dx_sum,
                        int act, float act_slope, void* stream);

/* ------------------------------------------------------------------------
 * The last per-point layer of a point-cloud model as ONE operator, forward and backward
 * (fusion rules table rows "Conv1d" and "BatchNorm1d", the element-wise rows, then the max over
 * points; section "Results" calls this workload memory-bound):
 *     pooled[b,n,c] = max_l act( BatchNorm_c( sum_ci W[b,c,ci] X[b,n,ci,l] + bias[b,c] ) )
 * The [Nb][B*Co][L] convolution output and its gradient are never formed, so no storage rounding
 * happens inside the operator.  bf16 storage only.  Device pointers throughout.
 *
 * Forward.  X (strides xs, unit point stride), W:[B][Co][Ci], bias:[B][Co] or NULL, gamma/beta and the
 * statistics arguments as in hfta_bn_fwd.  The batch statistics come from the moments of X
 * (mean_c = W_c E[x] + bias_c, var_c = W_c Cov(x) W_c^T, Cov from a Ci x Ci Gram matrix accumulated
 * in fp32 and combined in fp64); the maximum and its argmax from one pass of the matrix product.
 * Outputs: V (storage dtype) and idx (int32), both with strides vs; save_mean, save_invstd; updated
 * running statistics (if given); zhit fp32 [B][Nb][Co] = the convolution output at the argmax;
 * saved_moments fp32, hfta_conv1x1_bn_maxpool_saved_floats(B, Ci, Co) floats, or NULL: what the
 * backward can reuse (Gram matrix, sums of X, W times the Gram matrix).  idx is the lowest point
 * index that attains the maximum of the activated value, the maximum being decided on the fp32
 * matrix product (so against an exact evaluation the index can differ only where two points' values
 * lie within the product's rounding error, Ci * 2^-24 * sum_ci |W||X| scaled by |gamma| * invstd);
 * a row whose activated values are all equal (every point clipped by a ReLU, or gamma = 0) returns
 * index 0 and zhit at point 0.
 * act: NONE, RELU, or LEAKY with slope >= 0 (the argmax needs a non-decreasing activation).
 *
 * Backward.  Give exactly one of Z (the stored convolution output, strides zs, read ONLY at the
 * Nb*Co argmax points) or zhit; saved_moments from the forward or NULL (then recomputed here).
 * dV, idx, vs: pooled gradient and argmax.  Outputs dX (strides dxs, storage dtype), dW fp32
 * [B][Co][Ci], dbias fp32 [B][Co] or NULL (exactly zero: a bias in front of a BatchNorm), dgamma,
 * dbeta.  BatchNorm's backward is a per-channel affine map of z plus Nb spikes, so dX and dW reduce
 * to the Gram matrix of X, a Ci -> Ci product with the spikes added in, and gathers at the argmax.
 *
 * EUNSUPPORTED unless bf16, Ci <= 128, Ci % 8 == 0, Co <= 1024, L % 4 == 0 and L < 2^21, 8-byte
 * aligned X rows; EWORKSPACE below the *_workspace_bytes value (workspace 256-byte aligned; the
 * workspace-size functions return 0 for unsupported shapes).
 * ---------------------------------------------------------------------- */
size_t hfta_conv1x1_bn_maxpool_saved_floats(int B, int Ci, int Co);
size_t hfta_conv1x1_bn_maxpool_fwd_workspace_bytes(int B, int Nb, int Ci, int Co, int L, int dtype);
int hfta_conv1x1_bn_maxpool_fwd(int B, int Nb, int Ci, int Co, int L, int dtype,
                                const void* X, const int64_t xs[4], const void* W, const void* bias,
                                const float* gamma, const float* beta, float eps, float momentum,
                                float* running_mean, float* running_var, float* save_mean, float* save_invstd,
                                void* V, int32_t* idx, const int64_t vs[3], float* zhit, float* saved_moments,
                                int act, float act_slope, void* workspace, size_t ws_bytes, void* stream);
size_t hfta_conv1x1_bn_maxpool_bwd_workspace_bytes(int B, int Nb, int Ci, int Co, int L, int dtype);
int hfta_conv1x1_bn_maxpool_bwd(int B, int Nb, int Ci, int Co, int L, int dtype,
                                const void* X, const int64_t xs[4], const void* W, const void* bias,
                                const void* Z, const int64_t zs[4], const float* zhit, const float* saved_moments,
                                const void* dV, const int32_t* idx, const int64_t vs[3],
                                const float* gamma, const float* beta,
                                const float* save_mean, const float* save_invstd,
                                void* dX, const int64_t dxs[4], float* dW, float* dbias,
                                float* dgamma, float* dbeta, int act, float act_slope,
                                void* workspace, size_t ws_bytes, void* stream);

/* The same operator at the end of a chain of conv -> BatchNorm -> act blocks whose activated tensors
 * are not stored: X is given as the previous block's stored pre-activation Xpre with that block's
 * BatchNorm constants (in_gamma, in_beta, in_mean, in_invstd: [B][Ci] fp32; in_act in {NONE, RELU,
 * LEAKY}), and every kernel of the operator that reads X forms
 *   X = in_act(in_gamma (Xpre - in_mean) in_invstd + in_beta),  rounded to the storage dtype,
 * on load with the arithmetic of hfta_bn_fwd (see hfta_conv1x1_bn_prenorm_fwd).  Results are
 * bit-identical to storing X and calling the plain pair.  Shapes, workspaces, other arguments and
 * errors as the plain pair; the backward call takes the convolution output at the argmax (zhit),
 * not Z; dX is the gradient with respect to X.
 * Xact (optional, with strides xas[4], stride_l == 1, 8-byte aligned, strides % 4 == 0): the forward
 * operator's first kernel, which reads every element of Xpre exactly once, also writes X there, and
 * the operator's other kernels read X from it as the plain operator does.  The backward is then the
 * plain hfta_conv1x1_bn_maxpool_bwd on Xact.  This trades the on-load arithmetic in the two
 * kernels bound by their matrix products for one more tensor write; the normalisation pass of
 * the previous block (a read and a write of the tensor) is saved either way. */
int hfta_conv1x1_bn_maxpool_prenorm_fwd(int B, int Nb, int Ci, int Co, int L, int dtype,
                                        const void* Xpre, const int64_t xs[4],
                                        const float* in_gamma, const float* in_beta, const float* in_mean,
                                        const float* in_invstd, int in_act, float in_slope,
                                        const void* W, const void* bias, const float* gamma, const float* beta,
                                        float eps, float momentum, float* running_mean, float* running_var,
                                        float* save_mean, float* save_invstd,
                                        void* V, int32_t* idx, const int64_t vs[3], float* zhit, float* saved_moments,
                                        int act, float act_slope, void* Xact, const int64_t xas[4],
                                        void* workspace, size_t ws_bytes, void* stream);
int hfta_conv1x1_bn_maxpool_prenorm_bwd(int B, int Nb, int Ci, int Co, int L, int dtype,
                                        const void* Xpre, const int64_t xs[4],
                                        const float* in_gamma, const float* in_beta, const float* in_mean,
                                        const float* in_invstd, int in_act, float in_slope,
                                        const void* W, const void* bias, const float* zhit, const float* saved_moments,
                                        const void* dV, const int32_t* idx, const int64_t vs[3],
                                        const float* gamma, const float* beta,
                                        const float* save_mean, const float* save_invstd,
                                        void* dX, const int64_t dxs[4], float* dW, float* dbias,
                                        float* dgamma, float* dbeta, int act, float act_slope,
                                        void* workspace, size_t ws_bytes, void* stream);


/* ------------------------------------------------------------------------
 * Fused Adam over the parameter arena of all B models (section "Our Proposal:
 * HFTA", paragraph on optimizers: a vector of per-model learning rates applied
 * to the concatenated gradients).
 *   theta, m, v: fp32 [B][P], updated in place; grad: [B][P] in grad_dtype;
 *   theta_lowp: bf16 [B][P] copy of the new theta (NULL = none);
 *   lr, beta1, beta2, eps, weight_decay: fp32 [B] device arrays; step_t >= 1.
 *   g' = g + wd theta (decoupled_wd = 0)  or  theta *= 1 - lr wd first (decoupled_wd = 1)
 *   m = b1 m + (1-b1) g';  v = b2 v + (1-b2) g'^2
 *   theta -= lr (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps)
 * ---------------------------------------------------------------------- */
int hfta_adam_step(int B, int64_t P, int grad_dtype,
                   float* theta, const void* grad, float* m, float* v, void* theta_lowp,
                   const float* lr, const float* beta1, const float* beta2, const float* eps,
                   const float* weight_decay, int step_t, int decoupled_wd, void* stream);

/* The same update over a parameter-major arena, still ONE launch.  The fused model
 * keeps each fused parameter as its own tensor [B][n_j] (weights concatenated along
 * the model dimension, as the fusion rules table lays them out), and the arena is
 * those tensors back to back: fused parameter j occupies the flat element range
 * [B*seg_offsets[j], B*seg_offsets[j+1]) as [B][n_j], n_j = seg_offsets[j+1]-seg_offsets[j].
 *   seg_offsets: HOST array of nseg+1 per-model element offsets, seg_offsets[0] = 0,
 *   strictly increasing; nseg <= HFTA_ADAM_MAX_SEGMENTS.  theta, grad, m, v,
 *   theta_lowp: flat device buffers of B*seg_offsets[nseg] elements.
 *   B <= HFTA_ADAM_MAX_MODELS.  Everything else as hfta_adam_step. */
#define HFTA_ADAM_MAX_SEGMENTS 192
#define HFTA_ADAM_MAX_MODELS 1024
int hfta_adam_step_multi(int B, int nseg, const int64_t* seg_offsets, int grad_dtype,
                         float* theta, const void* grad, float* m, float* v, void* theta_lowp,
                         const float* lr, const float* beta1, const float* beta2, const float* eps,
                         const float* weight_decay, int step_t, int decoupled_wd, void* stream);

/* ------------------------------------------------------------------------
 * Fused Embedding and the core of fused multi-head attention (fusion rules table rows "Embedding":
 * one table of B*V rows with the indices of model b offset by b*V, here table [B][V][E] and indices
 * [B][R]; and "MultiheadAttention", which the table builds from the Linear rule: the input and
 * output projections are hfta_linear_fwd/bwd, the rest is per (model, sequence, head)).
 *   embedding_fwd: out[b,r,:] = scale * table[b, idx[b,r], :] (+ pos[r % S, :], fp32 [S][E], or NULL);
 *                  storage dtype; indices clamped to [0, V).
 *   embedding_bwd: dtable[b,v,:] (fp32, fully written) = scale * sum over r with idx[b,r] == v of dY[b,r,:],
 *                  added in order of r (bit-reproducible); R*8 bytes of LDS per workgroup: EUNSUPPORTED
 *                  above 7680 rows per model.
 *   attention_fwd: QKV [B][N][S][3E] = [q | k | v] per token, head h owns columns h*d..(h+1)*d of each
 *                  block (d = E/H).  P [B][N][H][S][S] (storage dtype) receives softmax(q k^T / sqrt(d))
 *                  (with causal != 0 entry [i][j] takes part only for j <= i, the rest is 0); CTX
 *                  [B][N][S][E] = P v, heads side by side.  No head split or transpose is materialised.
 *   attention_bwd: dQKV (same layout as QKV, fully written) from QKV, the saved P and dCTX; workspace
 *                  of hfta_attention_bwd_workspace_bytes (one score-sized buffer), else EWORKSPACE.
 * B*N*H <= 65535 (EUNSUPPORTED above); E must be a multiple of H (EINVAL).
 * ---------------------------------------------------------------------- */
/* Per-sample point transform of the point-cloud models (input / feature transform: a matrix
 * predicted per cloud and applied to all its points; the Linear / Conv1d rule with the weight indexed
 * by the sample as well as by the model).  X, Y, dY, dX: [b][n][c][l] with element strides (unit point
 * stride); T, dT: [B][Nb][Co][Ci] contiguous, storage dtype (T is an activation of the transform
 * sub-network, so its gradient is one too).
 *   fwd: Y[b,n,o,l] = sum_c T[b,n,o,c] X[b,n,c,l]
 *   bwd: dX[b,n,c,l] = sum_o T[b,n,o,c] dY[b,n,o,l] (NULL = skip);  dT[b,n,o,c] = sum_l dY[b,n,o,l] X[b,n,c,l] (NULL = skip)
 * One batched GEMM over (model, sample) each.  B*Nb <= 65535 (EUNSUPPORTED above). */
int hfta_point_transform_fwd(int B, int Nb, int Ci, int Co, int L, int dtype, const void* X, const int64_t xs[4],
                             const void* T, void* Y, const int64_t ys[4], void* stream);
int hfta_point_transform_bwd(int B, int Nb, int Ci, int Co, int L, int dtype, const void* X, const int64_t xs[4],
                             const void* T, const void* dY, const int64_t dys[4], void* dX, const int64_t dxs[4],
                             void* dT, void* stream);
/* hfta_softmax_xent for wide class axes (a vocabulary): one workgroup per row instead of one thread;
 * same results up to fp32 summation order; row terms pass through the workspace
 * (hfta_softmax_xent_rows_workspace_bytes, else EWORKSPACE) and are added per model in a fixed order. */
size_t hfta_softmax_xent_rows_workspace_bytes(int B, int R);
int hfta_softmax_xent_rows(int B, int R, int K, int dtype, const void* logits, const int32_t* labels,
                           float* loss, void* dlogits, void* workspace, size_t ws_bytes, void* stream);
int hfta_embedding_fwd(int B, int R, int V, int E, int dtype, const void* table, const int32_t* idx,
                       float scale, const float* pos, int S, void* out, void* stream);
int hfta_embedding_bwd(int B, int R, int V, int E, int dtype, const void* dY, const int32_t* idx,
                       float scale, float* dtable, void* stream);
int hfta_attention_fwd(int B, int N, int S, int E, int H, int dtype, const void* QKV, void* P, void* CTX,
                       int causal, void* stream);
size_t hfta_attention_bwd_workspace_bytes(int B, int N, int S, int E, int H, int dtype);
int hfta_attention_bwd(int B, int N, int S, int E, int H, int dtype, const void* QKV, const void* P,
                       const void* dCTX, void* dQKV, void* workspace, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Fused Adadelta over the same parameter-major arena, and the fused step learning-rate schedule
 * (section "Our Proposal: HFTA", paragraph on optimizers and learning-rate schedulers: each
 * hyper-parameter becomes a vector with one entry per model).  Arguments as hfta_adam_step_multi;
 * square_avg and acc_delta are the two fp32 state buffers; lr, rho, eps, weight_decay: device [B].
 *   g' = g + wd*theta;  v = rho v + (1-rho) g'^2;  d = sqrt(u + eps) / sqrt(v + eps) * g';
 *   u = rho u + (1-rho) d^2;  theta -= lr d
 * hfta_steplr: lr[b] = base_lr[b] * gamma[b] ^ floor(epoch / step_size[b]) (all device arrays of B
 * entries, step_size int32 >= 1; computed in double), so a schedule step is a launch on the
 * training stream and the optimisers read the result from device memory.
 * ---------------------------------------------------------------------- */
int hfta_adadelta_step_multi(int B, int nseg, const int64_t* seg_offsets, int grad_dtype,
                             float* theta, const void* grad, float* square_avg, float* acc_delta,
                             void* theta_lowp, const float* lr, const float* rho, const float* eps,
                             const float* weight_decay, void* stream);
int hfta_steplr(int B, const float* base_lr, const float* gamma, const int32_t* step_size, int epoch,
                float* lr, void* stream);

/* ------------------------------------------------------------------------
 * Support operators needed to close a training step (fusion rules table, rows
 * "ReLU", "LeakyReLU", "Tanh", "Dropout", "LayerNorm"; appendix "Fused Loss").
 * Elementwise operators work on `count` contiguous elements of any fused layout.
 * ---------------------------------------------------------------------- */
int hfta_act_fwd(int64_t count, int dtype, const void* X, void* Y, int act, float slope, void* stream);
/* dX = dY * act'(.)  `from_output` != 0: Z holds the activation OUTPUT (valid for
 * RELU, LEAKY with slope > 0, TANH); otherwise Z holds the pre-activation input. */
int hfta_act_bwd(int64_t count, int dtype, const void* Z, const void* dY, void* dX,
                 int act, float slope, int from_output, void* stream);
/* hfta_act_bwd (Z = pre-activation input) of a fused Linear's output [B][M][F] together with that
 * Linear's bias gradient (fusion rules table, Linear row: the bias gradient is the sum over the rows
 * of the output gradient): dX = dY * act'(Z) in the storage dtype and dbias[b][f] = sum over m of
 * dX[b][m][f] as stored (fp32 [B][F]), in one pass over the tensors.  Equals hfta_act_bwd followed by
 * hfta_linear_bwd's dbias up to fp32 summation order.  Device pointers, row-major, dX may alias dY.
 * EUNSUPPORTED unless F is a multiple of the 16-byte piece (8 bf16 / 4 fp32) and Z, dY, dX are
 * 16-byte aligned (use the two calls then); EINVAL on null pointers or non-positive sizes. */
int hfta_act_bwd_colsum(int B, int M, int F, int dtype, const void* Z, const void* dY, void* dX,
                        float* dbias, int act, float slope, void* stream);
/* Y = A + B element-wise over `count` elements of the storage dtype (the residual connection of
 * the MLP-block workload; fusion rules table, element-wise operators keep their shape with the
 * model dimension folded in).  Y may alias A or B.  Device pointers; EINVAL on null / count <= 0. */
int hfta_add(int64_t count, int dtype, const void* A, const void* B, void* Y, void* stream);
/* ------------------------------------------------------------------------
 * Pieces of a per-point (segmentation) head whose input is a concatenation of feature maps with a
 * tiled, point-independent part (the point-cloud segmentation workload of section "Methodology";
 * concatenation and tiling are element-wise in the model index, so they are expressed by strides:
 * a feature map is a channel slice of one [Nb][B*Ctot][L] buffer, nothing is copied).
 * Tensors are [b][n][c][l] with explicit element strides s[4] (unit point stride required) or
 * [b][n][c] with strides s[3]; storage dtype; device pointers; EINVAL on null / non-positive sizes.
 *   add_sample_bias: Y[b,n,c,l] = Z[b,n,c,l] + S[b,n,c]   (a k=1 convolution over [features | tiled
 *                    vector] = convolution over the features + the tiled part's product, once per sample)
 *   sum_points:      S[b,n,c] = sum_l X[b,n,c,l]           (its adjoint; fp32 accumulation, fixed order)
 *   add_strided:     Y = A + B element-wise                (gradient of a slice + gradient from the next layer)
 *   maxpool_points_bwd_add: dX[b,n,c,idx[b,n,c]] += dV[b,n,c] in place (hfta_maxpool_points_bwd added
 *                    onto an existing gradient; idx clamped to [0, L); dV, idx with strides vs)
 *   softmax_xent_points: scores [b][n][k][l], labels int32 [B][Nb][L]; per point softmax cross-entropy
 *                    over k; loss[b] (fp32) = mean over the model's Nb*L points; dlogits = its gradient.
 *                    Workspace: hfta_softmax_xent_points_workspace_bytes (EWORKSPACE below it).
 * Y may alias A (and Z).
 * ---------------------------------------------------------------------- */
int hfta_add_sample_bias(int B, int Nb, int C, int L, int dtype, const void* Z, const int64_t zs[4],
                         const void* S, const int64_t ss[3], void* Y, const int64_t ys[4], void* stream);
int hfta_sum_points(int B, int Nb, int C, int L, int dtype, const void* X, const int64_t xs[4],
                    void* S, const int64_t ss[3], void* stream);
int hfta_add_strided(int B, int Nb, int C, int L, int dtype, const void* A, const int64_t as[4],
                     const void* Bt, const int64_t bs[4], void* Y, const int64_t ys[4], void* stream);
int hfta_maxpool_points_bwd_add(int B, int Nb, int C, int L, int dtype, const void* dV, const int32_t* idx,
                                const int64_t vs[3], void* dX, const int64_t dxs[4], void* stream);
size_t hfta_softmax_xent_points_workspace_bytes(int B, int Nb, int L);
int hfta_softmax_xent_points(int B, int Nb, int K, int L, int dtype, const void* logits, const int64_t ls[4],
                             const int32_t* labels, float* loss, void* dlogits, const int64_t ds[4],
                             void* workspace, size_t ws_bytes, void* stream);

/* Adds a per-channel bias to an [Nb][K][HW] tensor (K = B*C channels) and applies act, in place. */
int hfta_bias_act_nchw(int64_t Nb, int64_t K, int64_t HW, int dtype, void* Y, const void* bias,
                       int act, float slope, void* stream);
/* Y = X * mask / (1-p); mask: uint8, 1 = keep; the same call is its own backward. */
int hfta_dropout(int64_t count, int dtype, const void* X, const uint8_t* mask, float p, void* Y,
                 void* stream);
/* LayerNorm over the last dim E of X:[B][R][E] with per-model affine w,b: fp32 [B][E]. */
int hfta_layernorm_fwd(int B, int R, int E, int dtype, const void* X, const float* w, const float* b,
                       float eps, float* save_mean, float* save_invstd, void* Y, void* stream);
size_t hfta_layernorm_bwd_workspace_bytes(int B, int R, int E);
int hfta_layernorm_bwd(int B, int R, int E, int dtype, const void* X, const void* dY, const float* w,
                       const float* save_mean, const float* save_invstd,
                       void* dX, float* dw, float* db, void* workspace, size_t ws_bytes, void* stream);
/* hfta_layernorm_bwd for a residual block y = LN(x + f(x)) (fusion rules table, LayerNorm and Linear
 * rows), with the two reductions that otherwise take passes of their own over [B][R][E]:
 *   the incoming gradient is dY + dY2 (dY2 may be NULL; the sum is rounded to the storage dtype as
 *   a stored element-wise sum would be), and
 *   dx_colsum[b][e] = sum over rows of dX[b][r][e] as stored (fp32 [B][E]): the bias gradient of the
 *   Linear whose output entered the LayerNorm's input.
 * Other arguments as hfta_layernorm_bwd; workspace hfta_layernorm_bwd_sums_workspace_bytes.
 * EUNSUPPORTED unless X, dY, dY2, dX are 16-byte aligned and E is a multiple of the 16-byte piece
 * with at most 128 pieces per row (use the separate calls then). */
size_t hfta_layernorm_bwd_sums_workspace_bytes(int B, int R, int E);
int hfta_layernorm_bwd_sums(int B, int R, int E, int dtype, const void* X, const void* dY, const void* dY2,
                            const float* w, const float* save_mean, const float* save_invstd,
                            void* dX, float* dw, float* db, float* dx_colsum,
                            void* workspace, size_t ws_bytes, void* stream);
/* Per-model losses with mean reduction over the model's own R rows; loss: fp32 [B];
 * dlogits in storage dtype.  No factor B appears because each model's loss is its
 * own mean (appendix "Fused Loss", eq. 3). */
int hfta_softmax_xent(int B, int R, int K, int dtype, const void* logits, const int32_t* labels,
                      float* loss, void* dlogits, void* stream);
int hfta_bce_logits(int B, int64_t R, int dtype, const void* logits, const void* targets,
                    float* loss, void* dlogits, void* stream);
/* The same for logits / targets / dlogits laid out by strides: element (b, r) at b*stride_b +
 * r*stride_r (a discriminator's [Nb][B] output is stride_b = 1, stride_r = B). */
int hfta_bce_logits_strided(int B, int64_t R, int dtype, const void* logits, const void* targets,
                            float* loss, void* dlogits, int64_t stride_b, int64_t stride_r,
                            void* stream);
int hfta_mse(int B, int64_t R, int dtype, const void* pred, const void* target,
             float* loss, void* dpred, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HFTA_H */
