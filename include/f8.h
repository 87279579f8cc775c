/*
 * f8 — 8-bit fixed-point inference layers for AMD MI355X (gfx950), C ABI.
 *
 * What a layer computes (F8Net, arXiv 2202.05239).  An 8-bit integer X with fractional
 * length FL stands for the real number X * 2^-FL (Sec. 3.1; word length 8 everywhere,
 * Sec. 4.3).  One layer is Eq. 6:  q_out = fix_quant( sum_j Weff_ij q_j + beff_i ),
 * fix_quant being Eq. 2 (unsigned, range 0..255, which is also the ReLU) or Eq. 9
 * (signed, range -127..127).  With q = X 2^-FL_x, Weff = W 2^-FL_w and the effective
 * bias held as a 32-bit integer B at the accumulator scale FL_x + FL_w this is
 *
 *     A      = sum_k X[k] * W[k] + B                      int8 x int8 -> int32
 *     A     += align(R)                                   optional residual (Sec. 4.3)
 *     Y      = clip( shift_round(A, s), clip_lo, clip_hi ),   s = FL_x + FL_w - FL_y
 *
 *     shift_round(a, s) = floor((a + 2^(s-1)) / 2^s)  for s >= 1   (round half up)
 *                       = a                           for s == 0
 *                       = a * 2^-s                    for s <  0
 *     align(r) = r * 2^d               for d = FL_x + FL_w - FL_res >= 0
 *              = shift_round(r, -d)    for d < 0
 *
 * Rescaling is the shift only: no 32-bit or floating-point multiply (Fig. 1(d), Sec. 1).
 * The result is one exactly defined integer tensor; the library reproduces it bit for
 * bit whatever tiling it uses, because integer addition is associative.
 *
 * Conventions for every entry point
 *   - Tensor pointers (x, w, bias, y, q->res, workspace) are DEVICE pointers owned by
 *     the caller; the struct pointers (q, layer descriptors) are HOST pointers read
 *     before the call returns.  Activations are NHWC, channel fastest.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *     enqueued asynchronously; the library does not synchronise (one exception below).
 *   - Arguments are validated on the host before anything is launched: a call that returns a
 *     validation error (anything but F8_ERR_DEVICE) has launched nothing.  Errors are status
 *     codes, never aborts.
 *   - Preconditions the library cannot check (they depend on device data): A and
 *     A + 2^(s-1) fit in int32 (the paper keeps accumulators in 32 bits, Sec. 4.3).
 *     K <= 65536 is enforced so that sum |X*W| alone cannot overflow; a bias large enough to
 *     break the precondition makes the accumulator wrap silently (two's complement), where the
 *     CPU oracle reports an overflow.  F8_ERR_ACC_OVERFLOW is reserved for checkers that see the data.
 *   - x, w, y must not overlap.  q->res may be any tensor of y's shape except y itself.
 *   - The single-layer dense calls keep a small device scratch buffer per (device, stream):
 *     256 bytes of zeros (the kernels' stand-in for padding) plus the folded accumulator
 *     start value, 4 bytes per output channel rounded up to 256 channels, at least 64 KiB.
 *     It is allocated (hipMalloc) on the first call on a stream and when a call needs more
 *     channels than any before it; growing waits for that stream first (the one place the
 *     library synchronises; such a call must not be made while the stream is being captured,
 *     and a graph that captured an earlier call keeps pointing at the freed buffer).
 *     f8_release_scratch() frees all of them.  Calls on different streams never share a buffer;
 *     calls on one stream are ordered by the stream, and the buffer's look-up and the two kernel
 *     launches of a call happen under one lock, so host threads may share a stream.
 *     f8_conv2d_fixed_ws (caller's workspace) and f8_conv2d_fixed_noalloc (a fixed array in the
 *     library) are the variants without this state.  The chain runner and the upstream steps
 *     allocate nothing: their memory is the caller's workspace.
 */
#ifndef F8_H
#define F8_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  F8_OK = 0,
  F8_ERR_NULL = 1,          /* a required pointer is NULL                                  */
  F8_ERR_SHAPE = 2,         /* a dimension is out of range (negative, K > 65536, ...)      */
  F8_ERR_FL = 3,            /* shift s outside [-8, 24] or residual shift outside [-24,24] */
  F8_ERR_CLIP = 4,          /* clip bounds outside the output type's range or lo > hi      */
  F8_ERR_DTYPE = 5,         /* type code not allowed for that operand                      */
  F8_ERR_ACC_OVERFLOW = 6,  /* reserved: reported by checkers that can see the data        */
  F8_ERR_ALIGN = 7,         /* int32 operand (bias, int32 y or residual) not 4-byte aligned */
  F8_ERR_UNSUPPORTED = 8,   /* valid but not implemented (tensor beyond 2^31-1 bytes, ...) */
  F8_ERR_DEVICE = 9,        /* the HIP runtime reported an error                           */
  F8_ERR_STATE = 10         /* chain used before f8_chain_prepare on that workspace        */
} f8_status;

typedef enum { F8_U8 = 0, F8_S8 = 1, F8_S32 = 2 } f8_dtype;

/* Per-call quantisation parameters (Eq. 2 / Eq. 9 / Eq. 6 in integer form). */
typedef struct {
  int32_t fl_x, fl_w, fl_y;   /* fractional lengths of input, weight and output             */
  int32_t clip_lo, clip_hi;   /* clip bounds in output LSBs (2^-fl_y).                      */
                              /* U8: 0 <= lo <= hi <= 255.  S8: -127 <= lo <= hi <= 127.    */
  int32_t x_type;             /* F8_U8 or F8_S8                                             */
  int32_t y_type;             /* F8_U8, F8_S8, or F8_S32 = write A itself (logits); then    */
                              /* fl_y and the clip bounds are ignored                       */
  const void *res;            /* device pointer: residual of y's shape, or NULL             */
  int32_t res_type;           /* F8_U8, F8_S8 or F8_S32                                     */
  int32_t fl_res;             /* fractional length of the residual                          */
} f8_quant;

/* Eq. 6 for a fully connected layer / 1x1 convolution.
 * x [M][K] 8-bit, w [N][K] int8, bias [N] int32 or NULL, y [M][N] (8-bit or int32). */
f8_status f8_gemm_fixed(const void *x, const int8_t *w, const int32_t *bias, void *y,
                        int M, int K, int N, const f8_quant *q, void *stream);

/* Eq. 6 for a convolution, implicit GEMM with M = B*P*Q, K = R*S*Cin, N = Cout.
 * x NHWC [B][H][W][Cin], w [Cout][R][S][Cin] int8, bias [Cout] or NULL,
 * y NHWC [B][P][Q][Cout], P = floor((H + 2 pad_h - R) / stride_h) + 1, Q likewise.
 * Padding is the real value 0. */
f8_status f8_conv2d_fixed(const void *x, const int8_t *w, const int32_t *bias, void *y,
                          int B, int H, int W, int Cin, int Cout, int R, int S,
                          int stride_h, int stride_w, int pad_h, int pad_w,
                          const f8_quant *q, void *stream);

/* f8_conv2d_fixed with the dense kernels' scratch supplied by the caller: the call keeps no state in
 * the library, allocates nothing, takes no lock and only enqueues kernels, so it can be captured
 * into a HIP graph and issued from any number of host threads and streams at once, as long as
 * calls that may overlap use different workspaces.  `workspace` is device memory, 256-byte
 * aligned, of at least f8_conv_workspace_bytes(Cout) bytes (F8_ERR_ALIGN / F8_ERR_SHAPE otherwise);
 * the call overwrites it (256 bytes of zeros, then the folded accumulator start values) and
 * later calls on the same stream may reuse it. */
size_t f8_conv_workspace_bytes(int Cout);
f8_status f8_conv2d_fixed_ws(const void *x, const int8_t *w, const int32_t *bias, void *y,
                             int B, int H, int W, int Cin, int Cout, int R, int S,
                             int stride_h, int stride_w, int pad_h, int pad_w,
                             const f8_quant *q, void *workspace, size_t workspace_bytes, void *stream);

/* f8_conv2d_fixed for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results, same
 * kernels; the only difference is where the dense kernels' scratch (256 bytes of zeros + the
 * folded accumulator start values, 4 bytes per output channel) lives: in a fixed array inside
 * the library's device code, (64 + F8_NOALLOC_MAX_COUT) * 4 bytes that every GPU the library
 * runs on holds until the process ends, instead of the per-stream hipMalloc'd buffer.  The call
 * never allocates, frees or synchronises.  Cout above F8_NOALLOC_MAX_COUT returns
 * F8_ERR_UNSUPPORTED before anything is launched.  All calls on one GPU share that one array
 * (each call rewrites the start values it needs; the zeros are never written): calls that may
 * overlap on one GPU (different streams, or several host threads) race; order them on one
 * stream. */
#define F8_NOALLOC_MAX_COUT 4096
f8_status f8_conv2d_fixed_noalloc(const void *x, const int8_t *w, const int32_t *bias, void *y,
                                  int B, int H, int W, int Cin, int Cout, int R, int S,
                                  int stride_h, int stride_w, int pad_h, int pad_w,
                                  const f8_quant *q, void *stream);

/* A second 8-bit format for the same accumulator (Sec. 4.3, "clipping-level sharing": the
 * children of one layer keep private fractional lengths, so the parent's 32-bit result is
 * quantised once per child format). */
typedef struct {
  int32_t fl_y;               /* fractional length of the second output                    */
  int32_t clip_lo, clip_hi;   /* its clip bounds in its own LSBs, same rules as f8_quant   */
  int32_t y_type;             /* F8_U8 or F8_S8                                            */
} f8_requant2;

/* f8_conv2d_fixed with two outputs: y as before, and
 *   y2 = clip(shift_round(A, fl_x + fl_w - q2->fl_y), q2->clip_lo, q2->clip_hi)
 * from the same A (bias and residual included), each with its own single rounding.  Both
 * outputs are 8-bit (q->y_type must not be F8_S32); y2 has y's shape, must not overlap y, x
 * or the residual.  The second shift obeys the same limits as the first (F8_ERR_FL). */
f8_status f8_conv2d_fixed_dual(const void *x, const int8_t *w, const int32_t *bias, void *y, void *y2,
                               int B, int H, int W, int Cin, int Cout, int R, int S,
                               int stride_h, int stride_w, int pad_h, int pad_w,
                               const f8_quant *q, const f8_requant2 *q2, void *stream);

/* Eq. 6 for a depthwise convolution (MobileNet V1/V2 layers of Sec. 5): K = R*S taps
 * per channel, no sum across channels.  x NHWC [B][H][W][C], w [R][S][C] int8,
 * bias [C] or NULL, y NHWC [B][P][Q][C]. */
f8_status f8_dwconv_fixed(const void *x, const int8_t *w, const int32_t *bias, void *y,
                          int B, int H, int W, int C, int R, int S,
                          int stride_h, int stride_w, int pad_h, int pad_w,
                          const f8_quant *q, void *stream);

/* Max pooling on 8-bit fixed-point activations (ResNet stem, Sec. 5 models).  The
 * quantiser of Eq. 2 is monotone, so the max of the integers is the quantised max and
 * the fractional length is unchanged.  Padding never wins; requires pad < window.
 * x NHWC [B][H][W][C], y NHWC [B][P][Q][C], both of type `dtype` (F8_U8 or F8_S8). */
f8_status f8_maxpool(const void *x, void *y, int B, int H, int W, int C, int R, int S,
                     int stride_h, int stride_w, int pad_h, int pad_w, int dtype, void *stream);

/* Global pooling as a fixed-point layer whose weights are all the integer 1 at
 * fractional length q->fl_w (the real weight 2^-fl_w):  y[b][c] = requant(sum_hw x).
 * With fl_w = ceil(log2(H*W)) and fl_y = fl_x this is the average up to the factor
 * 2^fl_w / (H*W), which belongs in the next layer's effective weights the way Eq. 6
 * absorbs every full-precision scale.  x NHWC [B][H][W][C], y [B][C].  H*W <= 65536.
 * q->res must be NULL. */
f8_status f8_global_pool_fixed(const void *x, void *y, int B, int H, int W, int C,
                               const f8_quant *q, void *stream);

/* ---- layer-chain runner: a whole fixed-point network forward (Sec. 5 models) ---- */

typedef enum { F8_OP_CONV = 0, F8_OP_DWCONV = 1, F8_OP_MAXPOOL = 2, F8_OP_GPOOL = 3 } f8_op;

/* One layer.  Tensors are numbered: 0 is the network input, layer i writes tensor
 * `dst` (> 0, each id written once, before it is read).  q.res is ignored; the residual
 * is the tensor `res` (or -1), whose type and fractional length go in q.res_type and
 * q.fl_res.  w and bias are device pointers that must stay valid while the chain lives. */
typedef struct {
  int32_t op;                       /* f8_op                                            */
  int32_t src, dst, res;            /* tensor ids; res = -1 for none                    */
  int32_t Cin, Cout, R, S;          /* pools: Cout == Cin; GPOOL ignores R,S            */
  int32_t stride_h, stride_w, pad_h, pad_w;
  f8_quant q;
  const int8_t *w;                  /* CONV [Cout][R][S][Cin]; DWCONV [R][S][C]; else NULL */
  const int32_t *bias;              /* [Cout] or NULL                                   */
  int32_t dst2;                     /* CONV only: id of a second output tensor in format q2
                                       (see f8_conv2d_fixed_dual), or <= 0 for none     */
  f8_requant2 q2;
} f8_layer_desc;

typedef struct f8_chain f8_chain;

/* Checks every layer (shapes, types and fractional lengths must chain), plans which
 * tensors share memory.  in_type is the type of tensor 0 (F8_U8 / F8_S8). */
f8_status f8_chain_create(const f8_layer_desc *layers, int n_layers, int in_h, int in_w,
                          int in_c, int in_type, f8_chain **out);
/* Bytes of device workspace needed for `batch` images (activations + folded constants). */
f8_status f8_chain_workspace_bytes(const f8_chain *c, int batch, size_t *bytes);
/* Writes the folded per-channel constants into the workspace; once per workspace and
 * batch size, before f8_chain_run. */
f8_status f8_chain_prepare(f8_chain *c, void *workspace, int batch, void *stream);
/* Runs all layers on x (tensor 0, NHWC, `batch` images); the last layer's output is
 * written to `out` (its own type; NHWC).  Must follow f8_chain_prepare with the same
 * workspace and batch.  Only kernel launches are enqueued, so the call can be captured
 * into a HIP graph. */
f8_status f8_chain_run(f8_chain *c, const void *x, void *out, void *workspace, int batch,
                       void *stream);
/* Where tensor `id` lives after a run (for per-layer checks): pointer inside the
 * workspace (or NULL for ids 0 and the last tensor), shape and type.  Tensors whose
 * memory was reused by a later layer are reported with *live_at_end = 0. */
f8_status f8_chain_tensor(const f8_chain *c, int id, void *workspace, int batch, void **ptr,
                          int *h, int *w, int *ch, int *dtype, int *live_at_end);
/* With keep_all != 0 no two tensors share memory (bigger workspace, every intermediate
 * can be inspected).  Call before f8_chain_workspace_bytes. */
f8_status f8_chain_set_keep_all(f8_chain *c, int keep_all);
/* Inverted-residual blocks (1x1 dense, 3x3 depthwise stride 1 pad 1, 1x1 dense, optional shortcut
 * from the block input; MobileNetV2, paper Sec. 5 and Appx) whose intermediate tensors have no other
 * reader can run as one kernel that keeps them on chip.  Same results; those tensors are then not
 * available through f8_chain_tensor.  Off by default (fusion = 1 switches it on; never used with
 * keep_all).  Call before f8_chain_workspace_bytes. */
f8_status f8_chain_set_fusion(f8_chain *c, int fusion);
/* n_streams = 2: f8_chain_run works on the two halves of the batch side by side, the first half on
 * the caller's stream and the second on a stream the chain owns (created here, default priority,
 * destroyed with the chain), which waits for what is already queued on the caller's stream and is
 * waited for by it at the end of the call: to the caller the call still behaves like work on one
 * stream, and it can still be captured into a HIP graph.  Images are independent (the layers of
 * Eq. 6 act on each image alone), so the results are the same; layers that leave part of the
 * chip idle, or that wait on memory, overlap with layers of the other half.  The workspace is
 * the same size.  Intermediate tensors are then not available through f8_chain_tensor; with
 * keep_all, or for a batch of one image, the call runs on one stream.  n_streams = 1 (the default)
 * turns it off. */
f8_status f8_chain_set_streams(f8_chain *c, int n_streams);
void f8_chain_destroy(f8_chain *c);

/* Measurement aids for the chain (not on the hot path).
 * f8_chain_layer_info: name of the kernel layer `layer` launches (copied into
 *   kernel_name, at most name_len bytes with the terminator) and the layer's algorithmic
 *   work for `batch` images: operations (2 per multiply-accumulate; 0 for pools) and
 *   bytes (every operand and result touched once).
 * f8_chain_profile: runs the chain 2 * `repeats` times with a HIP event recorded on
 *   `stream` before and after every layer, once with every layer launched once and once
 *   with every layer launched five times back to back; the difference divided by four is
 *   the duration of one launch in a busy stream (the cost of the event pair cancels).
 *   Waits for the stream and writes each layer's mean launch duration in milliseconds to
 *   layer_ms[f8_chain_num_layers].  The chain's output is the same as after f8_chain_run. */
int f8_chain_num_layers(const f8_chain *c);
f8_status f8_chain_layer_info(const f8_chain *c, int layer, int batch, char *kernel_name,
                              int name_len, double *alg_ops, double *alg_bytes);
f8_status f8_chain_profile(f8_chain *c, const void *x, void *out, void *workspace, int batch,
                           void *stream, int repeats, float *layer_ms);

/* ---- upstream of the integer layers: quantisers on real tensors, fractional-length choice,
 *      Conv-BN folding.  All tensors are device pointers to float32 unless said otherwise; every
 *      call only enqueues kernels on `stream` and allocates nothing.  `round` is round half up,
 *      as in the integer layers.  WL = 8 throughout. ---- */

/* Eq. 2 (unsigned, codes 0..255, 0 <= fl <= 8) and Eq. 9 (signed, codes -127..127, 0 <= fl <= 7):
 *   y[i] = 2^-fl * round(clip(x[i] * 2^fl, lo, hi)).
 * Exact in float32 (a power-of-two scaling, a clip, a rounding of a value below 2^8).  A NaN takes
 * the lower bound.  x and y may be the same buffer.  n = 0 is a no-op.  F8_ERR_FL for fl outside
 * the format's range, F8_ERR_ALIGN for pointers that are not 4-byte aligned (16-byte aligned
 * pointers take the vector path). */
f8_status f8_fix_quant_f32(const float *x, float *y, size_t n, int fl, int is_signed, void *stream);
/* The integer inside Eq. 2 / Eq. 9, as one byte per element (uint8 or int8): the input format of
 * the integer layers. */
f8_status f8_fix_quant_code(const float *x, void *q, size_t n, int fl, int is_signed, void *stream);
/* Eq. 3 with M = 255:  y = k_out * round(k_in * clip(x, 0, alpha)),  k_in = fl32(255 / alpha),
 * k_out = fl32(alpha / 255), every operation in float32 in that order.  alpha must be finite and
 * positive (F8_ERR_CLIP). */
f8_status f8_pact_f32(const float *x, float *y, size_t n, float alpha, void *stream);
/* Eq. 4: the same function written through the unsigned fix_quant,
 *   y = eta * fix_quant(x / eta),  eta = fl32(f8_eta_fix(alpha, fl)),
 * division, quantiser and product each in float32. */
f8_status f8_pact_fix_f32(const float *x, float *y, size_t n, float alpha, int fl, void *stream);
/* Eq. 5 (host): the fix scaling factor 2^fl * alpha / 255. */
double f8_eta_fix(double alpha, int fl);
/* Eq. 1 (host): floor(log2(40 / sigma)) for a signed tensor, floor(log2(70 / sigma)) for an
 * unsigned one, kept inside 0..7 / 0..8; sigma <= 0 (or NaN) gives the largest.  For an unsigned
 * (rectified) tensor sigma is that of the values before the rectifier (Sec. 3.1). */
int f8_opt_fl(double sigma, int is_signed);

/* Device scratch every reduction below needs: this many doubles, 8-byte aligned, contents
 * irrelevant before and after; calls that run concurrently need one each. */
#define F8_STATS_WORK_DOUBLES 4096
typedef struct {
  double mean, std;                 /* over all n elements; std is the population one (divide by n) */
  int32_t fl_signed, fl_unsigned;   /* Eq. 1 applied to std */
} f8_stats;
/* Statistics of a tensor for the fractional-length rule (Eq. 1), accumulated in fp64 about the
 * first element, in a fixed order (the result does not change from run to run).  `stats` is a
 * device pointer, written by the last kernel of the call.  n = 0 gives mean 0, std 0. */
f8_status f8_tensor_stats_f32(const float *x, size_t n, f8_stats *stats, double *work, void *stream);
/* The toy experiment of Sec. 3.1 (and the appendix on the statistical analysis) for one format:
 *   out[0] = sum |v - fix_quant(v)|,  out[1] = sum |v|,  out[2] = out[0] / out[1],
 * with v = x for the signed format and v = max(x, 0) for the unsigned one; out is a device
 * pointer to three doubles; sums in fp64 in a fixed order.  out[2] is NaN when every v is 0. */
f8_status f8_quant_error_f32(const float *x, size_t n, int fl, int is_signed, double *out, double *work,
                             void *stream);

/* Folding of one Conv-BN block into the integer layer's parameters (Eq. 6, Sec. 4.3).
 *   w      [cout][k] float32, k = R*S*Cin in the integer layer's weight order (k = R*S for a
 *          depthwise layer stored [C][R*S]; transpose to [R][S][C] is the caller's)
 *   gamma, beta, mu, sigma   [cout] float32: BN scale, shift, running mean, running standard
 *          deviation (sqrt(var + eps), formed by the caller).  A layer without BN passes
 *          gamma = sigma = 1, mu = 0, beta = its bias.
 *   eta_in, eta_out   fix scaling factors (Eq. 5) of this block's input quantiser and of its
 *          child's (the master child's where there are several); 1 for a tensor quantised by
 *          fix_quant directly
 *   fl_x   fractional length of the input activation codes
 *   fl_w   >= 0: fractional length of the weights; < 0: choose it by Eq. 1 from the standard
 *          deviation of the whole effective weight tensor (then `stats` must be given)
 * Computes, in fp64 with every operation rounded on its own and in this order,
 *   g_i = gamma_i / sigma_i,   scale_i = g_i * (eta_in / eta_out),   W_eff = w * scale_i,
 *   b_eff_i = (beta_i - g_i * mu_i) / eta_out,
 *   wq = round(clip(W_eff * 2^fl_w, -127, 127))             (Eq. 9, int8 [cout][k])
 *   bq = round(b_eff * 2^(fl_x + fl_w)) saturated to int32  (the accumulator's format)
 * and, if `stats` is not NULL, the statistics of W_eff with the chosen fl_w in stats->fl_signed.
 * wq, bq, stats and work are device pointers; work holds f8_fold_work_doubles(cout) doubles.
 * cout * k must stay below 2^31 (F8_ERR_SHAPE); eta must be finite and positive (F8_ERR_CLIP). */
typedef struct {
  int32_t cout, k;
  double eta_in, eta_out;
  int32_t fl_x, fl_w;
} f8_fold_desc;
size_t f8_fold_work_doubles(int cout);
f8_status f8_fold_conv_bn(const float *w, const float *gamma, const float *beta, const float *mu,
                          const float *sigma, const f8_fold_desc *d, int8_t *wq, int32_t *bq,
                          f8_stats *stats, double *work, void *stream);

/* ---- helpers (host side, set-up only) ---- */

/* A PACT clipping level alpha (Eq. 3) expressed in output LSBs for fractional length
 * fl_y: min(type max, round_half_up(alpha * 2^fl_y)), at least 0.  With the paper's
 * folding (Eq. 4-6) alpha is absorbed into the effective weights and the bound is the
 * full range; this helper serves callers that keep an explicit level. */
int32_t f8_clip_from_alpha(double alpha, int fl_y, int is_signed);
const char *f8_status_str(f8_status s);
/* Frees the per-stream scratch buffers of the single-layer calls (after the caller has
 * synchronised the streams that used them). */
void f8_release_scratch(void);
/* Measurement aid: plain streaming copy of `bytes` bytes (a multiple of 16; both device
 * pointers 16-byte aligned; the ranges must not overlap), 16 bytes per lane.  It is the
 * yardstick for what HBM delivers to a kernel that reads and writes every byte once, and the
 * known-size reference against which the memory-traffic counters are scaled. */
f8_status f8_copy_bytes(const void *src, void *dst, size_t bytes, void *stream);
/* Measurement aid: a register-only loop of the int8 matrix instruction the dense kernels use
 * (32x32x32, eight independent accumulators per wave, two waves per SIMD on every CU, no
 * memory traffic).  Its rate is the practical ceiling of the matrix cores, quoted next to the
 * published peak.  `sink` is a device buffer of at least F8_YARDSTICK_SINK_INTS ints (one
 * checksum per thread, contents meaningless); `iters` is the loop count per wave (1 .. 2^24);
 * *ops (host pointer, may be NULL) receives the operations one launch performs (2 per
 * multiply-accumulate). */
#define F8_YARDSTICK_SINK_INTS (512 * 256)
f8_status f8_mfma_i8_yardstick(int32_t *sink, int iters, double *ops, void *stream);
/* The same loop with chosen operands: seed 0 gives the loop above (a few small constants per lane),
 * any other seed fills every operand byte with pseudo-random bits, as real weights and activations
 * would.  The two rates differ on this chip: its clock under matrix load depends on how many
 * multiplier bits switch.  (Accumulators wrap; the sums mean nothing.) */
f8_status f8_mfma_i8_yardstick_operands(int32_t *sink, int iters, uint32_t seed, double *ops, void *stream);
/* Tuning switches: kernel choices only, never results (the parity tests force every tile variant
 * through them).  Names and defaults: "conv_variant" (-1 = automatic; >= 0 forces that tile
 * variant of the LDS-direct dense kernel), "conv_ws", "conv_ws_min" (768: smallest layer, in blocks
 * of 128 pixels, that takes the weights-stationary 3x3 kernel), "pw_ws", "pw_small", "xcd_remap",
 * "pw_wide", "pw_mid" (1: the 1x1 128 -> 512 kernel only together with the 512 -> 128 layer behind it, 2: also
 * alone), "stem_pool", "conv_tail", "conv_img" (1 = on), "conv_img_min" (96: fewest images, or
 * bands of 28 image rows, for which a chain takes the image-stationary 3x3 kernels).  The environment variables F8_<NAME IN CAPITALS> give the
 * initial values; they are read once, when the library first looks at a switch, never on the
 * launch path.  f8_tuning_set returns 0, or -1 for an unknown name; the chain switches
 * (the last four) are read by f8_chain_create.  f8_tuning_get returns the value (-1 for an unknown name). */
int f8_tuning_set(const char *name, int value);
int f8_tuning_get(const char *name);
/* Library version, for the binding to check that it loaded what it was built against. */
int f8_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif
