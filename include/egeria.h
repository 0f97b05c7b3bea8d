/*
 * libegeria: the plasticity-evaluation hot path of Egeria (arXiv 2201.06227)
 * for AMD Instinct MI355X (gfx950).
 *
 * For one layer module the path is (Section 4.1-4.2 of the paper):
 *   1. generate the reference model: quantise a snapshot of the training
 *      model's weights to int8                                (egeria_quantize*)
 *   2. run the reference model's forward on the same mini-batch and hook the
 *      module's output activation A_R                         (egeria_ref_forward)
 *   3. score the training model's activation A_T against A_R with the
 *      training-plasticity metric of Eq. 1 (SP loss)          (egeria_plasticity)
 * egeria_plasticity_eval chains 2 and 3 for a stack of modules,
 * egeria_refresh_eval chains 1, 2 and 3.
 *
 * General rules of this interface
 *   - Every pointer is a DEVICE pointer unless its comment says HOST.  The
 *     descriptor structs themselves are HOST memory holding device pointers.
 *   - The caller owns every buffer.  The library never allocates or frees
 *     device memory and never synchronises: work is enqueued on `stream` (a
 *     hipStream_t passed as void*; NULL is the default stream) and results
 *     land in device memory when the stream reaches them.  One exception to
 *     "on `stream`": for a stack of layers (n_layers > 1)
 *     egeria_plasticity_eval and egeria_refresh_eval enqueue the score of
 *     layer l on a side stream that the library creates once per device
 *     (default priority, on the device that is current at the first such
 *     call), ordered against `stream` with events in both directions; the
 *     side stream has joined `stream` again when the call returns, so
 *     whatever the caller enqueues on `stream` afterwards is ordered behind
 *     the whole call, and the call can be captured into a HIP graph.  The
 *     device of `stream` must be the current device.
 *   - Device pointers must be 16-byte aligned.
 *   - Argument errors are found on the host before anything is launched and
 *     are reported through the return code; nothing is thrown.
 *   - A NaN or infinity met by a quantiser sets a flag word inside the
 *     workspace; egeria_check reads it back (that call does synchronise).
 *   - Calls are re-entrant as long as they use distinct workspaces (host
 *     threads may call concurrently; the host-side enqueueing of stack
 *     evaluations, which share the device's side stream and its events, is
 *     serialised by a lock inside the library, and their scores then run one
 *     call after the other on that stream).  Two calls that share a workspace
 *     must be ordered on one stream.
 *
 * Quantisation rule (the paper names int8 post-training quantisation and
 * leaves the arithmetic to its framework; this library fixes it as):
 *   absmax = max |x_i|;  scale = fp32(absmax / 127);  inv = fp32(127 / absmax)
 *   (both divisions in fp64, rounded once); q_i = clamp(rne(x_i * inv), -127,
 *   127) with one fp32 multiply; zero point 0.  absmax == 0, or so small that
 *   inv overflows, quantises to all zeros with scale 1.  With a caller-supplied
 *   static scale: inv = fp32(1 / scale) and values beyond the range saturate.
 *
 * int8 operand layout: a quantised matrix [rows, K] is stored row-major with
 * each row padded with zero bytes to egeria_padded(K) = K rounded up to 16.
 * A quantised NHWC image tensor [B, H, W, C] pads C the same way.
 */
#ifndef EGERIA_H
#define EGERIA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    EGERIA_OK = 0,
    EGERIA_ERR_INVALID_ARG = 1,          /* null / misaligned pointer, non-positive size */
    EGERIA_ERR_UNSUPPORTED = 2,          /* valid request outside what the kernels cover */
    EGERIA_ERR_WORKSPACE_TOO_SMALL = 3,
    EGERIA_ERR_NONFINITE = 4,            /* reported by egeria_check only */
    EGERIA_ERR_HIP = 5                   /* a launch or runtime call failed */
} egeria_status;

typedef enum { EGERIA_F32 = 0, EGERIA_BF16 = 1 } egeria_dtype;

/* Precision of the reference model (Section 6.4 of the paper, Table 2: int8 by
 * default, float16 and float32 as the fallback when int8 fails).  At the float
 * precisions weights and every layer's input are rounded to nearest even to
 * that precision, products are summed in fp32 on the matrix cores, the epilogue
 * is y = act(sum + bias [+ block input as cast]) in fp32; there are no scales.
 * In a Transformer encoder layer the four linear layers (the ones the int8
 * reference quantises, Section 5) run at that precision; attention, GELU (erf
 * form, on the fp32 output of the first feed-forward layer) and the layer
 * norms take and give fp32 and are evaluated in fp64.  No static activation
 * scales, no per-channel scales. */
typedef enum { EGERIA_REF_INT8 = 0, EGERIA_REF_F16 = 1, EGERIA_REF_F32 = 2 } egeria_ref_precision;

/* Code of the activations of the int8 reference model.  Symmetric: codes in
 * [-127, 127], zero point 0, scale = absmax / 127 (the default, and what every
 * description above and below assumes).  Affine: the framework's default
 * activation code (Section 5 delegates the int8 arithmetic to the framework's
 * quantisation): uint8 codes with a zero point, from the extrema of the tensor,
 * every operation an IEEE fp32 one:
 *   hi = max(max x, 0), lo = min(min x, 0)
 *   scale = max((hi - lo) / 255, 2^-23);  zp = clamp(0 - rne(lo / scale), 0, 255)
 *   q = clamp(rne(x * (1 / scale)) + zp, 0, 255);  the value of a code is (q - zp) * scale.
 * Weights stay symmetric int8.  A layer multiplies the centred codes,
 * acc = sum_k (q_k - zp) * w_k (int32, exact; a padded 3x3 window pads the real
 * value zero, i.e. the centred code 0), and the epilogue is the symmetric one
 * with this acc and this scale.  In memory and at the observation points a
 * code is stored as the int8 value q - 128.  Affine codes need
 * egeria_qlinear.colsum; they exclude static activation scales and the float
 * reference precisions, and every quantise point costs two launches of its own
 * (no fused quantisers; the Transformer kinds take the fp64 attention of the
 * observed runs). */
typedef enum { EGERIA_ACT_SYMMETRIC = 0, EGERIA_ACT_AFFINE = 1 } egeria_act_scheme;

/* Kinds of layer module the reference forward knows. */
typedef enum {
    EGERIA_FC_RELU = 0,      /* y = ReLU(x W^T + bias)                                   */
    EGERIA_BASIC_BLOCK = 1,  /* conv3x3 - ReLU - conv3x3 (+ input) - ReLU                */
    EGERIA_BOTTLENECK = 2,   /* conv1x1 - ReLU - conv3x3 - ReLU - conv1x1 (+ input) - ReLU */
    EGERIA_BERT_LAYER = 3,   /* post-LN Transformer encoder layer                        */
    EGERIA_BERT_STACK = 4    /* n_layers such layers chained                             */
} egeria_block_kind;

/* HOST struct.  Shape of one layer module.
 *   FC_RELU     : batch, c_in (input features), c_out (output features)
 *   BASIC_BLOCK : batch, c_in = c_mid = c_out, height, width, has_residual
 *   BOTTLENECK  : batch, c_in, c_mid, c_out (= c_in when has_residual), height, width
 *   BERT_*      : batch, seq, hidden, heads, ffn, n_layers (1 for BERT_LAYER), ln_eps
 * Convolutions are stride 1; 3x3 ones use zero padding 1.  Batch-norm is taken
 * as folded into the convolution's weight and per-channel bias. */
typedef struct {
    int32_t kind;
    int32_t batch;
    int32_t c_in, c_mid, c_out;
    int32_t height, width;
    int32_t has_residual;
    int32_t seq, hidden, heads, ffn;
    int32_t n_layers;
    float ln_eps;
    int32_t ref_precision;          /* egeria_ref_precision; 0 = int8 */
    int32_t act_scheme;             /* egeria_act_scheme; 0 = symmetric */
} egeria_block_desc;

/* HOST struct.  One quantised linear / convolution layer of the reference model.
 *   w_q   : int8 [out, egeria_padded(K)]; K = in features for linear layers,
 *           K = kh*kw*egeria_padded(c_in) ordered (kh, kw, c) for convolutions
 *           (what egeria_quantize_nchw makes of an [out, in, kh, kw] tensor).
 *   scale : 1 fp32, the tensor's scale.
 *   bias  : fp32 [out] or NULL. */
typedef struct {
    const int8_t *w_q;              /* at a float reference precision: float16 / float32 values, rows padded
                                       to 16 bytes, as egeria_quantize_weights writes them; scale unused */
    const float *scale;             /* 1 fp32, or fp32 [out] when per_channel */
    const float *bias;
    int32_t per_channel;            /* 0: one scale for the tensor; 1: one per output channel */
    const int32_t *colsum;          /* affine activation codes only: what egeria_quantize_weights writes to
                                       egeria_weight.colsum for this tensor; else unused, may be NULL */
} egeria_qlinear;

/* HOST struct.  Affine parameters of one layer norm (each fp32 [hidden] or NULL
 * for gamma = 1 / beta = 0). */
typedef struct {
    const float *gamma;
    const float *beta;
} egeria_norm;

/* HOST struct.  The reference model of one layer module: `linear` in forward
 * order (FC: 1; BASIC: 2; BOTTLENECK: 3; BERT: per layer qkv, attn_out, ffn1,
 * ffn2), `norm` per BERT layer (post-attention, post-ffn); norm may be NULL. */
typedef struct {
    int32_t n_linear;
    const egeria_qlinear *linear;   /* HOST array */
    int32_t n_norm;
    const egeria_norm *norm;        /* HOST array or NULL */
    /* NULL: every activation is quantised with a dynamic scale (absolute maximum
     * of the tensor at run time).  Else a DEVICE array of n_linear fp32: the
     * static scale of the input of linear[i] (Section 5: static quantisation for
     * convolutional networks; values beyond 127 * scale saturate).  Scales must
     * be positive and finite.  FC and convolution kinds only; with the BERT kinds
     * (dynamic quantisation, Section 5) it is EGERIA_ERR_UNSUPPORTED.  In this
     * mode a layer that feeds another one writes that layer's int8 input
     * directly, without a fp32 round trip, and non-finite values are not
     * detected. */
    const float *act_scale;
} egeria_qweights;

/* HOST struct.  Optional observation points of the reference forward, used by
 * parity tests: for sub-layer i (same order as egeria_qweights.linear) the int8
 * input in the layout the GEMM consumes ([M, egeria_padded(K)], NHWC for
 * convolutions), its scale, the raw int32 accumulators [M, out] and the fp32
 * output after the epilogue [M, out].  Any pointer may be NULL.  At a float
 * reference precision x_q receives the cast operand rows (float16 / float32,
 * each row padded to 16 bytes), acc the bit patterns of the fp32 sums, x_scale
 * is not written.  With affine activation codes x_q receives q - 128, x_zp
 * (1 int32, else not written) the zero point, acc the sums of the centred codes. */
typedef struct {
    int8_t *x_q;
    float *x_scale;
    int32_t *acc;
    float *y;
    int32_t *x_zp;
} egeria_tap;

typedef struct {
    int32_t n;
    const egeria_tap *tap;          /* HOST array */
} egeria_taps;

/* K rounded up to a multiple of 16. */
int64_t egeria_padded(int64_t k);

/* Section 4.1: per-tensor int8 quantisation of n contiguous values (weights of
 * a snapshot, or any activation).
 *   x           n values of type dt.
 *   fixed_scale NULL: dynamic (scale from absmax); else 1 fp32 static scale.
 *   q           int8 [n] out.  scale_out: 1 fp32 out.
 *   ws          at least egeria_quantize_workspace_bytes() bytes.
 * n == 0 is valid and writes scale 1. */
egeria_status egeria_quantize(const void *x, egeria_dtype dt, int64_t n, const float *fixed_scale,
                              int8_t *q, float *scale_out, void *ws, size_t ws_bytes,
                              void *stream);

/* Same rule, for a matrix [rows, cols] whose quantised rows are padded:
 * q is int8 [rows, egeria_padded(cols)], pad bytes zero. */
egeria_status egeria_quantize_rows(const void *x, egeria_dtype dt, int64_t rows, int64_t cols,
                                   const float *fixed_scale, int8_t *q, float *scale_out,
                                   void *ws, size_t ws_bytes, void *stream);

/* Same rule, for an [n, c, h, w] tensor (a mini-batch of images, or a
 * convolution weight [out, in, kh, kw]) written channel-last:
 * q is int8 [n, h, w, egeria_padded(c)], pad channels zero. */
egeria_status egeria_quantize_nchw(const void *x, egeria_dtype dt, int64_t n, int64_t c, int64_t h,
                                   int64_t w, const float *fixed_scale, int8_t *q,
                                   float *scale_out, void *ws, size_t ws_bytes, void *stream);

/* HOST struct.  One weight tensor of a snapshot: a linear layer's [out, in]
 * matrix (kh = kw = 1) or a convolution's [out, in, kh, kw] kernel, contiguous. */
typedef struct {
    const void *w;
    int32_t dtype;                  /* egeria_dtype */
    int32_t out, in, kh, kw;
    int8_t *w_q;                    /* out: int8 [out, kh, kw, egeria_padded(in)], pad zero */
    float *scale;                   /* out: 1 fp32, or fp32 [out] when per_channel */
    int32_t per_channel;            /* 0: one scale for the tensor; 1: the same rule applied to every
                                       output channel w[o] on its own (one scale per channel) */
    int32_t precision;              /* egeria_ref_precision.  Float precisions: w_q receives float16 / float32
                                       values [out, kh, kw, cp], cp = `in` padded with zeros to a whole number of
                                       16-byte units (8 / 4 values); scale is not written and may be NULL */
    int32_t *colsum;                /* out, or NULL: sums of the int8 codes the affine activation codes need
                                       (egeria_act_scheme), int32 [classes, out]: for kh = kw = 1 one class, the
                                       sum over `in`; for a 3x3 kernel 16 classes, class c the sum over `in` and over
                                       the window positions that lie inside the image for an output pixel with
                                       (c & 1) first row, (c & 2) last row, (c & 4) first column, (c & 8) last column.
                                       int8 precision only */
} egeria_weight;

/* Section 4.1, reference-model generation: quantises all n weight tensors of
 * a snapshot, each with its own dynamic per-tensor scale, with the same codes
 * and scales egeria_quantize_rows / egeria_quantize_nchw give tensor by tensor,
 * in one or two kernel launches per 32 tensors.
 *   w   HOST array of n descriptors (device pointers inside).
 *   ws  at least egeria_quantize_weights_workspace_bytes(n) bytes.
 * Empty tensors are valid (scale 1).  Tensors of 2^31 or more padded bytes
 * are EGERIA_ERR_UNSUPPORTED. */
egeria_status egeria_quantize_weights(const egeria_weight *w, int32_t n, void *ws, size_t ws_bytes,
                                      void *stream);
size_t egeria_quantize_weights_workspace_bytes(int32_t n);

/* Section 4.1: the value an int8 code of the reference model stands for,
 * x_i = q_i * scale (one fp32 multiply).  q int8 [n], scale 1 fp32, x fp32 [n]
 * out; n == 0 is valid.  This is what a skip connection of the convolution
 * modules adds (the dequantised block input). */
egeria_status egeria_dequantize(const int8_t *q, const float *scale, int64_t n, float *x,
                                void *stream);

size_t egeria_quantize_workspace_bytes(void);

/* Affine uint8 codes of n contiguous values (egeria_act_scheme): q uint8
 * [egeria_padded(n)] (the bytes past n are written as zero), scale_out 1 fp32,
 * zp_out 1 int32.  ws at least
 * egeria_quantize_affine_workspace_bytes() bytes; n == 0 is valid (scale 2^-23,
 * zero point 0). */
egeria_status egeria_quantize_affine(const void *x, egeria_dtype dt, int64_t n, uint8_t *q, float *scale_out,
                                     int32_t *zp_out, void *ws, size_t ws_bytes, void *stream);
size_t egeria_quantize_affine_workspace_bytes(void);

/* Section 4.1 / 4.2: forward of the int8 reference model of one layer module on
 * the mini-batch x, producing the hooked activation A_R.
 *   x      fp32 mini-batch: [batch, c_in] (FC), NCHW [batch, c_in, h, w] (conv
 *          kinds), [batch, seq, hidden] (BERT kinds).
 *   a_ref  fp32 out, [n_layers][batch, D]: D = c_out (FC), h*w*c_out in NHWC
 *          order (conv kinds; the metric does not depend on the feature order),
 *          seq*hidden (BERT kinds).
 *   taps   NULL or observation points.  The int8 inputs, accumulators and
 *          intermediate outputs are defined only where a tap asks for them: a
 *          run without taps may keep them out of memory altogether (basic
 *          blocks of at most 16 channels quantise their operands while the
 *          convolutions load them), so the contents of ws after a call are
 *          unspecified apart from what egeria_check reads.  a_ref is the same
 *          bit for bit with and without taps.
 *   ws     at least egeria_workspace_bytes(desc) bytes.
 * Every linear / convolution input is quantised per tensor at run time
 * (dynamic scale), the contraction is int8 x int8 -> int32 on the matrix
 * cores, and the epilogue is, in fp32 and in this order: s = s_x * s_w;
 * y = fma((float)acc, s, bias); [+ residual]; activation.  The residual of the
 * conv kinds is the dequantised block input.
 * Transformer kinds (Section 5: dynamic quantisation, only the four linear
 * layers of a layer are int8): post-LN encoder layer, inference mode, no mask;
 * attention, layer norm and the erf-form GELU are floating point and are
 * evaluated so that every int8 code and scale of the following GEMM is the one
 * an fp64 evaluation rounded once to fp32 gives.  Limits of these kinds: x must
 * be EGERIA_F32 (a bf16 mini-batch is EGERIA_ERR_UNSUPPORTED), hidden / heads
 * <= 64 (larger heads: EGERIA_ERR_UNSUPPORTED), batch * seq < 2^31, at most 36
 * layers per stack; the score calls further need batch <= 128.
 * Errors: EGERIA_ERR_INVALID_ARG for a null or misaligned pointer, a bad
 * descriptor, n_linear / n_norm / taps->n that do not fit the module;
 * EGERIA_ERR_UNSUPPORTED as listed; EGERIA_ERR_WORKSPACE_TOO_SMALL. */
egeria_status egeria_ref_forward(const egeria_block_desc *desc, const egeria_qweights *qw,
                                 const void *x, egeria_dtype x_dt, float *a_ref,
                                 const egeria_taps *taps, void *ws, size_t ws_bytes, void *stream);

/* Section 4.2, Eq. 1: training plasticity P = SP_loss(A_T, A_R) of two
 * activations of the same mini-batch, both [b, D] row-major (sample-major):
 *   Gt = Q Q^T (b x b), G = rows of Gt divided by max(their L2 norm, 1e-12),
 *   P = sum_ij (G_T - G_R)_ij^2 / b^2.
 * p_out: 1 fp32.  ws: at least egeria_plasticity_workspace_bytes(b, D).
 * 1 <= b <= 128 (larger: EGERIA_ERR_UNSUPPORTED), D >= 1. */
egeria_status egeria_plasticity(const void *a_train, egeria_dtype t_dt, const void *a_ref,
                                egeria_dtype r_dt, int32_t b, int64_t D, float *p_out, void *ws,
                                size_t ws_bytes, void *stream);

size_t egeria_plasticity_workspace_bytes(int32_t b, int64_t D);

/* egeria_plasticity for callers that cannot allocate device memory and so have
 * no workspace to pass: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments (minus ws), same kernels
 * and the same result bit for bit; the scratch memory (ticket counter, row
 * shares, split-K partials) is a 16 MiB array inside the library's device
 * image, one copy per GPU, held until the process ends.  The call allocates
 * nothing and does not synchronise.
 * Limits: as egeria_plasticity, and egeria_plasticity_workspace_bytes(b, D)
 * must not exceed 16 MiB (EGERIA_ERR_UNSUPPORTED otherwise; every b <= 128 fits
 * on a 256-CU device).  All calls on one GPU share that GPU's array, which
 * keeps the previous call's contents (the kernels clear what must start at
 * zero): calls on one GPU that overlap in time - two streams, two threads -
 * race on it and give undefined scores; order them on one stream.  The device
 * of `stream` must be the current device. */
egeria_status egeria_plasticity_noalloc(const void *a_train, egeria_dtype t_dt, const void *a_ref,
                                        egeria_dtype r_dt, int32_t b, int64_t D, float *p_out,
                                        void *stream);

/* Sections 4.1-4.2, one plasticity evaluation: reference forward of a module
 * (or stack; Section 4.1, as egeria_ref_forward without observation points)
 * followed by one score per layer (Section 4.2, Eq. 1, as egeria_plasticity on
 * that layer's A_R, which stays inside the workspace):
 * a_train is a HOST array of desc->n_layers device pointers (each [batch, D] of
 * type t_dt), p_out receives n_layers fp32 scores.  ws: at least
 * egeria_workspace_bytes(desc) (which includes room for A_R and the metric). */
egeria_status egeria_plasticity_eval(const egeria_block_desc *desc, const egeria_qweights *qw,
                                     const void *x, egeria_dtype x_dt,
                                     const void *const *a_train, egeria_dtype t_dt, float *p_out,
                                     void *ws, size_t ws_bytes, void *stream);

/* Sections 4.1-4.2: refresh of the reference model and evaluation in one call.
 * The same as egeria_quantize_weights(w, n_w, ws_w, ws_w_bytes, stream) followed
 * by egeria_plasticity_eval(desc, qw, x, ..., ws, ws_bytes, stream), and the same
 * results bit for bit (qw must point at the tensors that w writes); passes over
 * the snapshot and over the mini-batch that do not depend on each other share
 * kernel launches (the snapshot's maxima with the mini-batch's maximum, the
 * snapshot's codes with the mini-batch's codes).  Arguments, ownership and
 * errors as for the two calls; nothing is enqueued if an argument of either is
 * rejected. */
egeria_status egeria_refresh_eval(const egeria_weight *w, int32_t n_w, void *ws_w, size_t ws_w_bytes,
                                  const egeria_block_desc *desc, const egeria_qweights *qw,
                                  const void *x, egeria_dtype x_dt,
                                  const void *const *a_train, egeria_dtype t_dt, float *p_out,
                                  void *ws, size_t ws_bytes, void *stream);

/* Host-only and pure: bytes of workspace egeria_ref_forward and
 * egeria_plasticity_eval need for this module; 0 if desc is invalid. */
size_t egeria_workspace_bytes(const egeria_block_desc *desc);

/* Section 4.1 leaves open what happens "if int8 fails"; the one failure this
 * library detects itself is a non-finite value at a quantiser (its scale would
 * be meaningless).  Reads the workspace's flag word back (synchronises `stream`): returns
 * EGERIA_ERR_NONFINITE if a quantiser that used this workspace met a NaN or
 * an infinity since the last check, and clears the flag. */
egeria_status egeria_check(void *ws, void *stream);

const char *egeria_status_string(egeria_status s);

/* ---- Freeze decision (Section 4.2 "How to Decide Layer Freezing", Eq. 2, Algorithm 1) ----
 * Host-only: consumes the stream of plasticity scores of the frontmost active
 * layer module and says when to freeze it and when to unfreeze everything.
 * Nothing here touches the GPU.
 *
 * Per evaluation (egeria_freeze_observe), in the algorithm's order:
 *   1. If the front module is the last one, nothing is decided.
 *   2. If fewer than W consecutive stale evaluations have been counted: the score
 *      is smoothed (Eq. 2, read as the mean of the last min(W, count) scores),
 *      appended to the module's history, the least-squares slope s of the last
 *      min(max(W, 2), length) smoothed values against 0, 1, 2, ... is taken (no
 *      slope from a single value: the counter is reset), and the counter is incremented if
 *      |s| < T, else reset.  With T <= 0 at init, T is 20 % of the largest |s|
 *      among the module's first three slopes and nothing is counted before.
 *      Otherwise the module is frozen: action FREEZE, the next module becomes
 *      the front with empty history (the score passed in is ignored).
 *   3. With lr_annealing set: once lr <= 0.1 * lr_ref * (1 + 1e-12), lr_ref being
 *      the rate passed in when the first module was frozen, every module is
 *      unfrozen, the first becomes the front again and W is halved (integer
 *      division, at least 1): action UNFREEZE_ALL.
 * All arithmetic is fp64.  W must be in [1, EGERIA_FREEZE_MAX_W]. */
#define EGERIA_FREEZE_MAX_W 256

typedef enum { EGERIA_FREEZE_NONE = 0, EGERIA_FREEZE_FREEZE = 1, EGERIA_FREEZE_UNFREEZE_ALL = 2 } egeria_freeze_action;

/* HOST struct, owned by the caller, initialised by egeria_freeze_init; its
 * fields are the controller's whole state (no hidden allocation). */
typedef struct {
    int32_t n_modules, front, W, stale, lr_annealing, has_lr_ref, n_first_slopes, has_T;
    int64_t n_raw, n_smooth;                 /* values seen for the front module */
    double T_user, T, max_first_slope, lr_ref;
    double raw[EGERIA_FREEZE_MAX_W];         /* ring: last W scores */
    double smooth[EGERIA_FREEZE_MAX_W];      /* ring: last W smoothed scores */
} egeria_freeze_state;

/* HOST struct.  What one evaluation decided.  smoothed / slope are NaN when the
 * evaluation produced none (freeze call, last module, first value). */
typedef struct {
    int32_t action;                          /* egeria_freeze_action */
    int32_t front;                           /* frontmost active module after this evaluation */
    int32_t stale;                           /* consecutive stale evaluations counted so far */
    int32_t W;                               /* current window / counter length */
    double smoothed, slope, T;               /* T is NaN until known */
} egeria_freeze_decision;

egeria_status egeria_freeze_init(egeria_freeze_state *st, int32_t n_modules, int32_t W, double T,
                                 int32_t lr_annealing);
egeria_status egeria_freeze_observe(egeria_freeze_state *st, double p, double lr,
                                    egeria_freeze_decision *out);

/* ---------------------------------------------------------------------------
 * Activation cache (Section 4.3 of the paper, "Caching frozen layers'
 * activations", Figure 6): a table in GPU memory whose key is the sample id and
 * whose value is that sample's activation at the last frozen layer.  The
 * activations of coming mini-batches are put in ahead of the forward pass
 * (egeria_cache_put; where they come from - storage, an earlier epoch - is the
 * caller's business), the forward pass of the active layers reads them back by
 * sample id (egeria_cache_get), and only the most recent `window` mini-batches
 * are kept (five in the paper).
 *
 * Semantics: a put makes its mini-batch the newest one; when `window`
 * mini-batches are already held the oldest is dropped with its samples, except
 * those that a newer mini-batch has put in again (they are served from the
 * newer one).  An id that occurs twice in one put keeps its last row.  Negative
 * ids are not samples: never stored, never found.  A get copies the row of
 * every id that is held to out[i] and sets hit[i] = 1; for the others hit[i] = 0
 * and out[i] is left untouched.
 *
 * The cache lives in caller-owned DEVICE memory of egeria_cache_bytes(desc)
 * bytes (header, ids of the window * batch row slots, an open-addressing table
 * of at least twice that many entries rebuilt by every put, the rows
 * themselves), 16-byte aligned.  egeria_cache_init must run once before the
 * first put.  Calls on one cache must be ordered on one stream; nothing
 * synchronises, the put counter lives in the cache's own memory, so all three
 * calls can be captured into a HIP graph.
 * Limits: 1 <= window, 1 <= batch <= 65535, window * batch <= 2^20, row_elems >= 1;
 * a put takes at most `batch` ids, a get at most 65535.  ids, rows, out and hit are
 * DEVICE pointers; rows and out are [n, row_elems] row-major of type `dtype`.
 * Errors: EGERIA_ERR_INVALID_ARG for a bad descriptor, a null or misaligned
 * pointer or n out of range; EGERIA_ERR_WORKSPACE_TOO_SMALL when cache_bytes is
 * below egeria_cache_bytes(desc).
 * ------------------------------------------------------------------------- */
typedef struct {
    int32_t window;        /* mini-batches kept */
    int32_t batch;         /* most samples one put may bring */
    int64_t row_elems;     /* elements of one sample's activation */
    int32_t dtype;         /* egeria_dtype of the rows */
} egeria_cache_desc;

size_t egeria_cache_bytes(const egeria_cache_desc *desc);                       /* 0 for a bad descriptor */
egeria_status egeria_cache_init(const egeria_cache_desc *desc, void *cache, size_t cache_bytes, void *stream);
egeria_status egeria_cache_put(const egeria_cache_desc *desc, void *cache, size_t cache_bytes,
                               const int64_t *ids, int32_t n, const void *rows, void *stream);
egeria_status egeria_cache_get(const egeria_cache_desc *desc, const void *cache, size_t cache_bytes,
                               const int64_t *ids, int64_t n, void *out, uint8_t *hit, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* EGERIA_H */
