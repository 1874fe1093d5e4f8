/*
 * libclt -- one training step of a cross-layer transcoder (CLT) on one AMD
 * MI355X (gfx950).  C ABI: plain pointers and sizes, no C++ or framework types.
 *
 * The model (paper Sec. 2.1): per layer l an encoder with JumpReLU,
 *     pre[l] = x[l] W_enc[l] + b_enc[l],   z[l] = pre[l] * 1[pre[l] > theta[l]]   (eq. 1)
 * and a cross-layer decode in which target layer l' sums the contributions of
 * all source layers l <= l',
 *     y_hat[l'] = sum_{l <= l'} z[l] W_dec[p(l,l')] + b_dec[l']                    (eq. 3)
 * trained on the objective of App. B (reconstruction + lambda0 * tanh sparsity
 * weighted by the decoder norm + lambda1 * dead-feature penalty, see clt_loss)
 * with Adam (App. C, Table 1).
 *
 * Tensors (all DEVICE pointers owned by the caller, contiguous, row-major,
 * 16-byte aligned; the library never allocates, frees or keeps them):
 *   x      [L,B,d]  MLP inputs      storage type T (see clt_config.dtype), or int8 codes
 *   y      [L,B,d]  MLP outputs     T, or int8 codes
 *   W_enc  [L,d,F]  T               b_enc [L,F] float     theta [L,F] float
 *   W_dec  [P,F,d]  T, P = L(L+1)/2 b_dec [L,d] float
 *   z, pre [L,B,F]  T               y_hat [L,B,d] float (always fp32)
 *   act_class [L,B,F] uint8: bit 0 = active (pre > theta), bit 1 = inside the
 *          straight-through window |pre - theta| < ste_bandwidth/2, bit 2 = below
 *          the threshold (pre < theta strictly: where the dead-feature penalty of
 *          App. B has a gradient); all three decided on the fp32 accumulator
 *          before any rounding.  With the TopK activation only bit 0 is used.
 * Packed decoder: block p(l,l') = l*L - l(l-1)/2 + (l'-l), 0 <= l <= l' < L
 * (source-major: all decoders that leave source layer l are contiguous, which
 * is the "concatenation" whose row norm the sparsity term uses); each block is
 * [F,d] row-major, so one feature's decoder row is contiguous.
 * The vectors b_enc, theta, b_dec, their gradients and all Adam moments are
 * always float; T applies to the matrices and activations.
 *
 * Every function returns 0 (CLT_OK) or a negative clt_status.  Arguments are
 * checked before any kernel is launched; after an error nothing was enqueued.
 * All work is enqueued on the caller's HIP stream (`stream` is a hipStream_t
 * passed as void*; NULL = the default stream) and the functions do not
 * synchronise, except clt_loss when asked for a host copy of the loss.
 * Calls on one handle must not overlap (they share its workspace).
 *
 * Environment switches, read at every call, for comparison runs and tests only
 * (each selects the slower of two kernels that compute the same thing):
 *   CLT_NO_XCD_PACING  the decode GEMM without the per-XCD pacing of its K segments
 *   CLT_GDZ_NO_LDS     list-driven dz: one wave per entry instead of d y_hat rows staged in LDS
 *   CLT_SD_ROWS        list-driven dW_dec: whole rows per workgroup instead of eight column slices
 *   CLT_NO_FUSED_DZ    list-driven dz as a kernel of its own even where the dW_dec kernel could take it
 */
#ifndef CLT_H_
#define CLT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct clt_handle clt_handle;

typedef enum clt_status {
  CLT_OK = 0,
  CLT_ERR_INVALID_ARG = -1, /* null pointer, bad enum or scalar               */
  CLT_ERR_SHAPE = -2,       /* L,d,F,B out of the supported range              */
  CLT_ERR_ALIGN = -3,       /* a tensor pointer is not 16-byte aligned         */
  CLT_ERR_WORKSPACE = -4,   /* workspace missing, misaligned or too small      */
  CLT_ERR_HIP = -5,         /* a HIP runtime call failed (see clt_last_error)  */
  CLT_ERR_STATE = -6        /* calls out of order (loss before forward, ...)   */
} clt_status;

enum { CLT_DTYPE_F32 = 0, CLT_DTYPE_BF16 = 1 };
enum { CLT_INPUT_NATIVE = 0, CLT_INPUT_INT8_ROWSCALE = 1 };
enum { CLT_DECODE_AUTO = 0, CLT_DECODE_DENSE = 1, CLT_DECODE_GATHER = 2 };
enum { CLT_ACT_JUMPRELU = 0, CLT_ACT_TOPK = 1 };

/* Plain data; set .size = sizeof(clt_config).  Shapes: L >= 1, B >= 1,
 * d and F positive multiples of 8. */
typedef struct clt_config {
  uint32_t size;
  int32_t L, d, F, B;
  int32_t dtype;          /* CLT_DTYPE_F32: fp32 storage and fp32 FMA accumulate;
                             CLT_DTYPE_BF16: bf16 storage, bf16 MFMA, fp32 accumulate */
  int32_t input_format;   /* CLT_INPUT_INT8_ROWSCALE: x and y are int8 codes with one
                             float scale per (layer, token) row (Sec. 3.1 cache format) */
  int32_t master_weights; /* 1: clt_adam_step updates fp32 master copies of W_enc/W_dec  */
  int32_t decode_mode;    /* dense GEMMs, active-feature gather kernels (Sec. 3.2: the decode, and here
                             also the two backward contractions through the decoder), or chosen per
                             step, on the device, from the measured density                        */
  int32_t log_threshold;  /* 0: the theta tensor holds the threshold itself; 1: it holds
                             tau = log(theta) (App. B writes the threshold as exp(tau)), the
                             kernels take exp() of it and theta's gradient and Adam step are
                             those of tau                                                   */
  int32_t activation;     /* CLT_ACT_JUMPRELU (eq. 1's z = pre 1[pre > theta]) or CLT_ACT_TOPK (Sec. 3.2
                             names it): per token and layer the topk_k largest pre-activations are
                             kept (z = pre there, the lower feature index wins among equal values),
                             decided on the fp32 pre-activation.  With TopK the theta tensor is
                             ignored by every call, its gradient is 0 and lambda1 must be 0.       */
  int32_t topk_k;         /* 0 <= topk_k <= F; read only when activation == CLT_ACT_TOPK           */
  int32_t reuse_decoder_norms; /* 0: every clt_forward computes the decoder norms (App. B) from W_dec.
                             1: a training loop that owns its weights may skip that pass over W_dec: a
                             clt_backward_adam_step that updates W_dec inside its weight-gradient kernel
                             (bf16, any decode mode, F and d multiples of 256) also leaves the row sums of
                             squares of the UPDATED weights, and the next clt_forward on this handle
                             that is given the same W_dec pointer forms the norms from them.  The
                             caller promises that nothing else writes W_dec between those two calls.
                             Whenever the sums are not there, clt_forward reads W_dec as with 0.      */
  float gather_density_threshold; /* AUTO: the forward decode gathers when the mean active
                             fraction of the batch is <= this and no (layer, token) row has
                             more than about 32x the larger of the two thresholds in listed
                             features (else the step decodes densely; the backward is not
                             bound by that row limit where d is a multiple of 32).  On an MI355X the
                             gather decode breaks even with the dense one near 0.005
                             (38-44 active of 8192 features; binding default 0.0045).    */
  float list_backward_density_threshold; /* AUTO: the backward through the decoder (dz, dW_dec
                             and its Adam update) runs on the active-feature lists when the
                             mean active fraction is <= this (same row limit); 0 = the same
                             as gather_density_threshold.  The list-driven backward pays up
                             to a higher density than the gather decode: it breaks even
                             near 0.02 (about 165 of 8192), whatever the expansion factor
                             (the dense cost grows with F, the list-driven one with the
                             active count); binding default 0.016.  The workspace holds room
                             for the partial sums of dz sized from this threshold (at most
                             320 listed entries per token and layer); a step whose lists are
                             longer goes backward through the dense kernels.                */
  float C;                /* sparsity scale C of the App. B objective                     */
  float ste_bandwidth;    /* width eps of the rectangle kernel of the threshold gradient */
  float beta1, beta2, adam_eps; /* Adam (App. C Table 1: 0.9, 0.999)                     */
} clt_config;

/* The five learned tensors, or things shaped like them (gradients, moments). */
typedef struct clt_tensors {
  void* W_enc;  /* [L,d,F] */
  float* b_enc; /* [L,F]   */
  float* theta; /* [L,F]   */
  void* W_dec;  /* [P,F,d] */
  float* b_dec; /* [L,d]   */
} clt_tensors;

/* Bytes of device workspace clt_init needs for this configuration. */
int clt_workspace_bytes(const clt_config* cfg, size_t* bytes);

/* Creates a handle bound to `workspace` (device memory, 256-byte aligned, at
 * least clt_workspace_bytes long, owned by the caller and kept alive until
 * clt_destroy).  Fails with CLT_ERR_HIP when no HIP device is usable. */
int clt_init(clt_handle** handle, const clt_config* cfg, void* workspace, size_t workspace_bytes);
int clt_destroy(clt_handle* handle);

/* Message of the last error on this handle (or of the last failed clt_init /
 * clt_workspace_bytes on this thread when handle is NULL).  Never NULL. */
const char* clt_last_error(const clt_handle* handle);

/* Activation normalisation (Sec. 3.1, last paragraph): every activation is
 * divided by a per-layer factor c[l], the mean L2 norm of that layer's token
 * vectors over the first batches, so that norms come out near one.  Inputs
 * and targets each have their own factors (call once per side).
 *
 * clt_norm_accumulate adds, for every layer, the sum over the B rows of
 * ||a[l,b,:]||_2 to norm_sum[l] (device, [L] double, 16-byte aligned; the
 * caller zeroes it before the first batch and counts the tokens).  a is
 * [L,B,d] in the handle's input format; a_scale [L,B] for int8 rows (the norm
 * of the codes times |scale|), else NULL.  Deterministic (fixed order). */
int clt_norm_accumulate(clt_handle* handle, void* stream, const void* a, const float* a_scale, double* norm_sum);

/* clt_norm_accumulate for callers that cannot allocate device memory or bring a
 * workspace (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): no handle, no workspace, and the call allocates nothing.
 * Same kernels and same result, bit for bit, as clt_norm_accumulate; the
 * per-block partial sums live in a 512 KB array that the library itself holds
 * on every GPU it runs on until the process ends.  Limit: L * ceil(B / 32) <=
 * 65536 partial sums (e.g. L = 16 with up to 131072 tokens per call), beyond
 * it the call fails with CLT_ERR_WORKSPACE; 1 <= L <= 128, d a positive
 * multiple of 8; dtype / input_format as in clt_config (a is [L,B,d] in that
 * format, a_scale [L,B] exactly when the rows are int8 codes).  The array's
 * address is looked up on the first call on a device (or by clt_init): make
 * that call before any graph capture.  Nothing in the array has to be cleared
 * between calls (every partial sum a call reads it has written first), but all
 * calls on one GPU share it: calls that overlap on one GPU, on different
 * streams or threads, race and must be serialised by the caller. */
int clt_norm_accumulate_static(void* stream, int32_t L, int32_t B, int32_t d, int32_t dtype, int32_t input_format,
                               const void* a, const float* a_scale, double* norm_sum);

/* Divides by c[l] = norm_sum[l] / n_tokens.  int8 rows: the division folds
 * into the dequantisation scale, scale_out[l,b] = scale_in[l,b] / c[l]
 * (scale_out may be scale_in), the codes are untouched and a_in, a_out must be
 * NULL.  Native rows: a_out = a_in / c[l] (a_out may be a_in), scales NULL.
 * A layer whose norm_sum is 0 (all-zero activations) is left unscaled. */
int clt_normalise(clt_handle* handle, void* stream, const double* norm_sum, int64_t n_tokens,
                  const void* a_in, const float* scale_in, void* a_out, float* scale_out);

/* Encoder + JumpReLU (eq. 1), decoder norms (App. B), cross-layer decode (eq. 3).
 * x_scale: [L,B] float for int8 inputs, else NULL.  Outputs: z, act_class,
 * y_hat are required; pre and l0_per_layer ([L] int32, active entries per
 * layer summed over tokens) may be NULL. */
int clt_forward(clt_handle* handle, void* stream,
                const void* x, const float* x_scale,
                const void* W_enc, const float* b_enc, const float* theta,
                const void* W_dec, const float* b_dec,
                void* z, void* pre, uint8_t* act_class, float* y_hat, int32_t* l0_per_layer);

/* App. B objective, mean over the B tokens:
 *   L_rec  = (1/B) sum (y_hat - y)^2,
 *   L_sp   = (lambda0/B) sum tanh(C z n[l,f]),
 *   L_dead = (lambda1/B) sum ReLU(theta[l,f] - pre[l,b,f]) n[l,f]   (dead-feature penalty).
 * Needs the decoder norms of the preceding clt_forward on this handle.  pre is
 * the pre-activation that clt_forward wrote and theta the threshold tensor as
 * given to it; both may be NULL when lambda1 == 0 (term off, nothing read).
 * Writes loss_dev[0..3] = {L_rec + L_sp + L_dead, L_rec, L_sp, L_dead} (device)
 * and keeps d y_hat and the decoder-norm gradient column sums in the workspace
 * for clt_backward.  If loss_host is not NULL the four floats are also copied
 * there and the stream is synchronised. */
int clt_loss(clt_handle* handle, void* stream,
             const void* y, const float* y_scale, const float* y_hat, const void* z,
             const void* pre, const float* theta,
             float lambda0, float lambda1, float* loss_dev, float* loss_host);

/* Backward pass of the App. B objective through eq. 3 and eq. 1 (chain rule;
 * the paper leaves it to autograd): gradients of the objective evaluated by the
 * preceding clt_loss, w.r.t. the five learned tensors (grads->W_enc, W_dec in T;
 * vectors float).  JumpReLU passes gradient to pre where active; theta gets the
 * rectangle-kernel pseudo-gradient -(theta/eps) sum_b 1[in window] dz.  With
 * lambda1 > 0 the dead-feature term adds -(lambda1/B) n to d pre and +(lambda1/B) n to d theta
 * for every entry with pre < theta, and its decoder-norm derivative to dW_dec.
 * With log_threshold the theta gradient is the one w.r.t. tau (times theta).
 * When the preceding clt_forward decoded through the active-feature lists, dz and
 * dW_dec are computed from those lists as well (same sums, zero terms skipped). */
int clt_backward(clt_handle* handle, void* stream,
                 const void* x, const float* x_scale, const float* theta,
                 const void* W_dec, const void* z, const uint8_t* act_class,
                 const clt_tensors* grads);

/* One Adam step (App. C Table 1: betas 0.9 / 0.999, learning rate 2e-4 there;
 * 1-based step count t, bias correction on, eps outside the square root, no
 * weight decay) on all five tensors.  m and v hold float moments for every
 * tensor.  master: NULL, or fp32 master copies of W_enc and
 * W_dec (its vector members are ignored) that are updated and then rounded
 * into params. */
int clt_adam_step(clt_handle* handle, void* stream, int64_t t, float lr,
                  const clt_tensors* params, const clt_tensors* grads,
                  const clt_tensors* m, const clt_tensors* v, const clt_tensors* master);

/* clt_backward (App. B objective) and clt_adam_step (App. C Table 1) in one
 * call, with the Adam update of W_enc and W_dec fused into the epilogues of the
 * two weight-gradient GEMMs (same update rule, applied to the fp32
 * accumulators): the matrix gradients are never stored
 * unless grads->W_enc / grads->W_dec are given, and the weight, moment and master
 * traffic of the optimiser runs under the contractions instead of after them.
 * theta and W_dec are taken from params.  grads->b_enc, theta, b_dec are required
 * (the vectors go through the separate Adam kernel).  Results equal the two
 * separate calls except that the matrix gradients enter Adam in fp32 instead of
 * after rounding to T. */
int clt_backward_adam_step(clt_handle* handle, void* stream,
                           const void* x, const float* x_scale, const void* z, const uint8_t* act_class,
                           int64_t t, float lr, const clt_tensors* params, const clt_tensors* grads,
                           const clt_tensors* m, const clt_tensors* v, const clt_tensors* master);

/* Device pointers into the workspace, for inspection by tests and tools:
 * which = 0 decoder norms [L,F] float; 1 d y_hat [L,B,d] T; 2 d pre [L,B,F] T
 * (with int8 inputs every row holds d pre times that row's x_scale: the form
 * the encoder-weight gradient contracts with the integer codes);
 * 3 sparsity column sums G [L,F] float; 4 decode switch, 4 int32: {what the measured
 * density allows: bit 0 the gather decode, bit 1 the list-driven backward through the
 * decoder (the backward clears it again when the lists turn out too long for it),
 * bit 2 that this backward works without the per-(layer, token) lists;
 * longest (layer, token) list, active and in-window features; path taken by the last
 * forward (1 dense, 2 gather); longest per-layer total of the feature lists, written by
 * the backward when it runs on the lists}; gather and auto decode modes only.
 * Valid after the call that writes them. */
int clt_workspace_view(const clt_handle* handle, int which, void** ptr, size_t* bytes);

/* Optional per-kernel timing, for benchmarks and profiling (not part of the
 * method).  While enabled, every kernel the library enqueues is bracketed by
 * HIP events on the caller's stream.  clt_profile_query waits for the recorded
 * events and returns, for kernel index 0 <= kernel < clt_profile_num_kernels(),
 * its name (static string), the accumulated device milliseconds and the number
 * of launches since profiling was last enabled. */
int clt_profile_enable(clt_handle* handle, int on);
int clt_profile_num_kernels(void);
int clt_profile_query(clt_handle* handle, int kernel, const char** name, double* total_ms, int64_t* launches);

/* Diagnostic, not part of the method: the instruction stream of the bf16
 * contraction kernels (one workgroup of 8 wavefronts per compute unit, per
 * iteration 64 v_mfma_f32_16x16x32_bf16 per wavefront), taken apart to show
 * what the matrix cores sustain on this board and what each kind of data
 * movement costs them.  The bf16 MFMA rate is limited by board power, and the
 * power depends on the operand bits, so every variant runs on all-zero or on
 * pseudo-random data.  mode is a sum of
 *    1  pseudo-random data instead of zeros
 *    2  MFMA operands are read from LDS (twelve 16-byte reads per lane for every
 *       32 MFMAs, the contraction kernels' pattern) instead of held in registers
 *    4  eight 16-byte LDS writes per lane and iteration (staging of a 256x64 + 64x256 tile)
 *    8  eight 16-byte loads per lane and iteration (64 KB per workgroup) from a
 *       region that stays in the L2
 *   16  (with 8) every second of those loads from a region that only fits the
 *       Infinity Cache
 *   32  the arrangement of a kernel with ONE wavefront per SIMD instead: 4
 *       wavefronts per compute unit, each with 8x8 accumulators, sixteen LDS
 *       reads for 64 MFMAs (2/3 of the LDS read traffic), 128 MFMAs per
 *       wavefront and iteration
 *   64  (with 32 + 8) the staging goes global memory -> LDS directly instead of
 *       through registers and LDS writes
 *  128  (alone) the bare loop on the other bf16 shape, 32 v_mfma_f32_32x32x16_bf16
 *       per wavefront and iteration: the same flop with four times the
 *       accumulator registers read and written per instruction
 * Built combinations: 0, 2, 6, 14, 30, 8, 24, 32, 34, 38, 46, 62, 110, 126, 128 (+1).  There is no data flow between
 * the parts and no barrier: the kernel computes nothing, it only does the work.
 * Enqueues on `stream` (a fill of buf first when a load bit is set); the caller
 * times it.  buf: device scratch, 16-byte aligned, at least (64 KB + 512 KB) x
 * compute units bytes when a load bit is set, else ignored.  counters_dev:
 * device, 4 x uint64, 16-byte aligned; after the kernel [0] holds the shader
 * cycles and [1] the ticks of the constant-rate counter that one wavefront
 * spent in its loop (shader clock = [0] / [1] * wall_clock_hz).  *flop (host)
 * receives the floating-point operations of the launch, *wall_clock_hz the
 * counter's rate; both may be NULL. */
int clt_diag_mfma_loop(void* stream, int iters, int mode, void* buf, size_t buf_bytes, uint64_t* counters_dev,
                       double* flop, double* wall_clock_hz);

#ifdef __cplusplus
}
#endif
#endif /* CLT_H_ */
