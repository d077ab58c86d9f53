/*
 * dit.h -- C ABI of the MI355X (gfx950) Diffuse-stage library.
 *
 * The library runs the denoising loop of a diffusion pipeline's Diffuse stage
 * (paper section 2.1):  eps_t = eps_theta(x_t, t, c);  x_{t-1} = Phi(x_t, t, eps_t),
 * T times from Gaussian x_T, where eps_theta is a diffusion transformer evaluated on the
 * latent tokens joined with the condition tokens (paper section 1: the noise is
 * concatenated with c).  A call serves a batch of requests of different resolutions
 * packed back to back (the paper's requests range over resolutions and durations,
 * appendix D workload table).
 *
 * Conventions for every entry point
 *  - "dev" pointers are device (HBM) addresses on the device given to dit_create; "host"
 *    pointers are ordinary host memory.  The library never allocates or frees device
 *    memory: weights, workspace, latents and conditions are the caller's buffers.
 *  - All GPU work is enqueued on the HIP stream given to dit_create (or dit_set_stream).
 *    dit_get_tensor / dit_set_tensor / dit_profile_read block until their copies are done.
 *    dit_denoise_step and dit_sample return without waiting for the GPU, with one exception:
 *    the FIRST of them after dit_bind, dit_init_weights or dit_set_tensor waits for the
 *    stream and reads the q/k norm gains back (a few KB, see dit_bind) before it launches.
 *    The dit_op_* calls stage their small host arrays with hipMemcpyAsync from pageable
 *    memory, which returns only after the host data has been read.
 *  - Every call returns a dit_status; arguments are validated before anything is
 *    launched, so a failing call leaves the caller's buffers untouched.  The text of the
 *    last error is kept per context (dit_last_error).  Nothing aborts or throws.
 *  - A context is not thread-safe; different contexts are independent.
 */
#ifndef DIT_H
#define DIT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dit_ctx dit_ctx;

typedef enum {
  DIT_OK = 0,
  DIT_EINVAL = 1,       /* null pointer, bad enum, bad scalar                          */
  DIT_ESHAPE = 2,       /* dimensions inconsistent with the configuration              */
  DIT_ENOMEM = 3,       /* weight arena or workspace smaller than required             */
  DIT_EDEVICE = 4,      /* a HIP call failed                                           */
  DIT_EUNSUPPORTED = 5, /* valid but not implemented (listed per function)             */
  DIT_ENOTFOUND = 6     /* unknown tensor or tap name                                  */
} dit_status;

/* Block families of eps_theta (the paper leaves the inside of the model open; these are
 * the three architectures of the benchmark configurations). */
enum { DIT_FAMILY_J = 0, /* joint two-stream blocks, absolute 2-D sin/cos positions      */
       DIT_FAMILY_F = 1, /* double-stream then single-stream blocks, rotary positions    */
       DIT_FAMILY_W = 2  /* self-attention + cross-attention + MLP, rotary positions     */ };

enum { DIT_UPDATE_EULER = 0, /* x <- x + (sigma_next - sigma_cur) v  (flow matching)     */
       DIT_UPDATE_DDIM = 1   /* deterministic DDIM with alpha_bar = 1 - sigma^2           */ };

typedef struct {
  int family;                 /* DIT_FAMILY_*                                            */
  int n_blocks;               /* J, W: blocks; F: double-stream blocks                   */
  int n_single;               /* F: single-stream blocks; otherwise 0                    */
  int hidden;                 /* d; multiple of 256                                      */
  int n_heads, head_dim;      /* hidden == n_heads*head_dim; head_dim is 64 or 128       */
  int mlp_hidden;             /* multiple of 256                                         */
  int latent_ch;              /* C                                                       */
  int patch_t, patch_h, patch_w;
  int cond_dim;               /* width of the condition tokens, multiple of 64           */
  int rope_axes[3];           /* rotary widths for (frame,row,col); all 0 = no rotary    */
  float rope_theta;
  int act_dtype;              /* DIT_ACT_*: storage type of activations between kernels  */
} dit_config;

/* Activation storage.  Only bf16 is built: GEMM and attention operands are bf16 MFMA inputs,
 * while accumulators, softmax and norm statistics, the residual stream, the model output and
 * the latent are float32 in either mode.  dit_create returns DIT_EUNSUPPORTED for
 * DIT_ACT_F32 (an all-float32 debug mode of the smallest benchmark configuration). */
enum { DIT_ACT_F32 = 0, DIT_ACT_BF16 = 1 };

/* One request: latent extent in LATENT units and number of condition tokens. */
typedef struct { int frames, height, width, n_cond; } dit_req;

/* ---- life cycle -------------------------------------------------------------------- */

/* Validates cfg and builds the host-side tensor table.  Makes no HIP call, so it also
 * works where no GPU is present.  `hip_stream` is a hipStream_t (may be NULL = default
 * stream).  On failure *out is NULL. */
dit_status dit_create(const dit_config* cfg, int device, void* hip_stream, dit_ctx** out);
void       dit_destroy(dit_ctx* ctx);
dit_status dit_set_stream(dit_ctx* ctx, void* hip_stream);
const char* dit_last_error(const dit_ctx* ctx);

/* Bytes of the weight arena (bf16 matrices stored [out][in] with padded leading
 * dimension, fp32 vectors), and of the workspace for a batch and at most `max_steps`
 * steps per dit_sample call (conditioning vectors of all steps are computed up front).
 * dit_workspace_bytes returns 0 on invalid requests.  Limits of one call (DIT_ESHAPE beyond
 * them): 4096 requests, 2^20 tokens, and tokens x max(3*hidden, hidden + mlp_hidden) < 2^31
 * (activation matrices are indexed with 32-bit element offsets). */
size_t dit_weight_bytes(const dit_ctx* ctx);
size_t dit_workspace_bytes(const dit_ctx* ctx, int n_req, const dit_req* reqs, int max_steps);

/* How the self-attention launch of a request list is cut up (host arithmetic only, no device call):
 * out[0] queries per workgroup (128 or 256), out[1] query blocks per head, out[2] how many of these
 * blocks run as key-split shares and out[3] the number of shares each (1: none).  Blocks are split
 * when all requests have one shape, the head count is a multiple of 8 and the last round of
 * workgroups would fill less than three quarters of the chip (Appendix "Impact of Batch Size" times
 * exactly such same-shape batches); the shares' partial sums live in the workspace, are added in a
 * fixed order, and only the form of attention without a running maximum (bounded q/k-norm gains)
 * uses them.  DIT_ATTN_SPLIT=0 in the environment switches the splitting off. */
dit_status dit_attention_plan(const dit_ctx* ctx, int n_req, const dit_req* reqs, int out[4]);

/* Hands the caller's device buffers to the context (both 256-byte aligned).  The
 * workspace may be re-bound at any time; its contents carry nothing between calls.  The
 * library keeps a host copy of the largest |gain| of every q/k norm (it bounds the attention
 * logits), refreshed on the first step after dit_bind, dit_init_weights or dit_set_tensor: a
 * caller that writes the arena by other means calls dit_bind again afterwards. */
dit_status dit_bind(dit_ctx* ctx, void* dev_weights, size_t weight_bytes,
                    void* dev_workspace, size_t workspace_bytes);

/* ---- weights ------------------------------------------------------------------------ */

/* Fills the bound arena: matrices and tables ~ N(0, std^2) rounded to bf16, biases 0,
 * norm gains 1.  Element i (row-major index in the logical [in][out] matrix) of tensor
 * `name` is std * g(seed, name, i) with g the counter-based Gaussian of the benchmark's
 * input recipe: key = mix(seed ^ fnv1a64(name)*PHI), z = mix(key + i),
 * g = sqrt(-2 ln u1) cos(2 pi u2) in float64 from the top 24 and next 24 bits of z. */
dit_status dit_init_weights(dit_ctx* ctx, uint64_t seed, float std);

/* Tensor table.  kind: 0 matrix [in][out], 1 bias [out], 2 norm gain, 3 table [rows][out].
 * For vectors `rows_in` is 1. */
int        dit_tensor_count(const dit_ctx* ctx);
dit_status dit_tensor_info(const dit_ctx* ctx, int index, char* name_buf, size_t name_buf_len,
                           int* rows_in, int* cols_out, int* kind);

/* Copies one tensor between the arena and host float32 in logical row-major [in][out]
 * order; n must equal rows_in*cols_out.  Matrices are rounded to bf16 on upload. */
dit_status dit_set_tensor(dit_ctx* ctx, const char* name, const float* host_src, size_t n);
dit_status dit_get_tensor(dit_ctx* ctx, const char* name, float* host_dst, size_t n);

/* ---- the hot path ------------------------------------------------------------------- */

/* One denoising step for n_req packed requests (paper section 2.1 equation).
 *  latents   dev, float32, IN/OUT: request r holds [C][frames][height][width], requests
 *            back to back.
 *  cond      dev, bf16: request r holds [n_cond][cond_dim], back to back; read-only.
 *  sigma_cur, sigma_next   host float32 [n_req]: noise level of this step and the next
 *            per request; the model sees t = 1000*sigma_cur.
 *  update_kind  DIT_UPDATE_*.  DDIM needs sigma_cur < 1.
 *  v_out     dev float32, same layout as latents, receives eps_theta's output; may be NULL.
 * Frames/height/width must be divisible by the patch; family J needs frames == 1. */
dit_status dit_denoise_step(dit_ctx* ctx, int n_req, const dit_req* reqs, float* latents,
                            const void* cond, const float* sigma_cur, const float* sigma_next,
                            int update_kind, float* v_out);

/* T steps.  sigmas: host float32 [n_req][T+1], row r = sigma_0 ... sigma_T of request r.
 * Equivalent to T calls of dit_denoise_step, but step-invariant work (condition
 * projection, conditioning vectors of every step, position tables) is done once.
 * At most 4 calls may be in flight on the stream: a fifth call waits for the first one's
 * host-to-device parameter copies.
 * T must not exceed the max_steps the workspace was sized for. */
dit_status dit_sample(dit_ctx* ctx, int n_req, const dit_req* reqs, float* latents,
                      const void* cond, const float* sigmas, int T, int update_kind);

/* ---- test and measurement hooks ----------------------------------------------------- */

/* Registers a capture: when the next steps reach the named point its tensor is copied
 * (device to device, on the stream) into dev_dst.  Points: "x_txt0", "x_img0",
 * "<blk>.q", "<blk>.k", "<blk>.attn", "<blk>.<stream>.ln1", "<blk>.<stream>.qkv",
 * "<blk>.<stream>.x_attn", "<blk>.<stream>.mlp_act", "<blk>.<stream>.x_out", "final"
 * with <blk> = blk<l> | dbl<l> | sgl<l> and <stream> = txt | img ("<blk>.q" holds the
 * queries as the attention kernel reads them: multiplied by log2(e)/sqrt(head_dim)).
 * `bytes` is the capacity
 * of dev_dst; a smaller tensor is copied whole, a larger one fails the step with
 * DIT_ENOMEM.  dit_tap_info reports rows/cols/element size of the last capture. */
dit_status dit_set_tap(dit_ctx* ctx, const char* point, void* dev_dst, size_t bytes);
dit_status dit_tap_info(const dit_ctx* ctx, const char* point, int* rows, int* cols, int* elem_bytes);
void       dit_clear_taps(dit_ctx* ctx);

/* Per-kernel-class timing with HIP events on the context's stream.  While enabled every
 * launch of the step is bracketed by an event pair; dit_profile_read synchronises the
 * stream and returns, per class, the summed milliseconds and launch count since the last
 * dit_profile_enable(ctx, 1).  Classes: 0 gemm, 1 attention, 2 layer-norm/modulate,
 * 3 q/k norm + rotary + V transpose, 4 latent update, 5 other. */
enum { DIT_PROF_GEMM = 0, DIT_PROF_ATTN = 1, DIT_PROF_LNMOD = 2, DIT_PROF_QKNORM = 3,
       DIT_PROF_UPDATE = 4, DIT_PROF_OTHER = 5, DIT_PROF_NCLASS = 6 };
dit_status dit_profile_enable(dit_ctx* ctx, int on);
dit_status dit_profile_read(dit_ctx* ctx, int klass, double* total_ms, long long* launches,
                            double* flop, double* bytes);

/* ---- single operations (the kernels of the step, callable alone) -------------------- */

/* C = A * W^T (+ bias) on MFMA.  A: dev bf16 [M][lda]; W: dev bf16 [N_pad][ldw] with N_pad
 * a multiple of 256 rows readable; bias: dev float32 [N] or NULL; K multiple of 64.
 * out_kind 0: bf16 [M][ldc];  1: float32 [M][ldc];  2: bf16 of tanh-GELU(acc + bias);
 * 3: float32 residual  out[m][n] += gate[row_req[m]*gate_stride + n] * (acc + bias),
 *    gate/row_req may be NULL (gate 1).  `stream` NULL = default stream. */
dit_status dit_op_gemm(void* stream, const void* A, int lda, const void* W, int ldw,
                       const float* bias, int M, int N, int K, int out_kind, void* out, int ldc,
                       const float* gate, int gate_stride, const int* row_req);

/* As dit_op_gemm (out_kind 0..2 only) with the tile variant forced, for tuning sweeps:
 * BM*1000+BN in {256256, 256128, 128256, 128128}; +1000000 = 8 waves (256256 only);
 * +10000000 / +20000000 = k-slab 32 with a 4- / 5-stage LDS ring instead of k-slab 64 with
 * 2 stages (256256, 1256256, 128128); 30128128 = 128x128 with k-slab 64 and a 4-stage ring. */
dit_status dit_op_gemm_variant(void* stream, const void* A, int lda, const void* W, int ldw,
                               const float* bias, int M, int N, int K, int out_kind, void* out,
                               int ldc, int variant);

/* The QKV product with its q/k epilogue, as the denoising step runs it when no capture point
 * is registered: C = A W^T + bias; output columns [0, nq) are queries, [nq, nq+nk) keys, the
 * rest is written as bf16 to out[M][ldc] at its own column (out is not written for q/k
 * columns).  Per row and head (head_dim 64 or 128 consecutive columns): x <- x / sqrt(mean(x^2)
 * + 1e-6) * gain, adjacent pairs (2j, 2j+1) rotated by the (cos, sin) in rope[dst][head_dim/2]
 * (dev float32 pairs, row = destination row; NULL = no rotation), queries times qscale; the
 * result goes as bf16 to qo / ko (dev, row stride ldo) at row dst_row[m] (dev int32, NULL =
 * m) and the column inside the q (k) range.  nq, nk multiples of 256; qgain/kgain dev
 * float32 [head_dim]. */
dit_status dit_op_gemm_qknorm(void* stream, const void* A, int lda, const void* W, int ldw,
                              const float* bias, int M, int N, int K, void* out, int ldc,
                              int nq, int nk, int head_dim, const float* qgain, const float* kgain,
                              const float* rope, const int* dst_row, void* qo, void* ko, int ldo,
                              float qscale);

/* As dit_op_gemm, computed as `splits` partial products over disjoint shares of K (each a
 * whole number of 64-wide slabs, 1 <= splits <= K/64) that a second kernel sums in fixed
 * order before the epilogue: the form the denoising step uses when M is small (few tiles,
 * long K).  work: dev scratch of at least ceil(M/128)*ceil(N/128)*splits*65536 bytes. */
dit_status dit_op_gemm_splitk(void* stream, const void* A, int lda, const void* W, int ldw,
                              const float* bias, int M, int N, int K, int out_kind, void* out,
                              int ldc, const float* gate, int gate_stride, const int* row_req,
                              int splits, void* work, size_t work_bytes);

/* dit_op_gemm_splitk for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels and the
 * same result bit for bit, with the partial tiles kept in an array inside the library's own
 * device image instead of a caller-supplied `work` buffer.  The call allocates and frees
 * nothing.  Limit: ceil(M/128)*ceil(N/128)*splits*65536 <= DIT_STATIC_SCRATCH_BYTES (16 MiB,
 * i.e. 256 partial tiles; each GPU the library runs on holds this array until the process
 * ends); larger products return DIT_ENOMEM before anything is launched.  The array belongs to
 * the device that is current at the call and is shared by every call on that device: calls
 * that overlap on one GPU (different streams, different threads) race on it and must be
 * serialised by the caller.  Nothing in it needs clearing between calls: each call's product
 * kernel writes every partial tile its reduction reads. */
#define DIT_STATIC_SCRATCH_BYTES (16u << 20)
dit_status dit_op_gemm_splitk_static(void* stream, const void* A, int lda, const void* W, int ldw,
                                     const float* bias, int M, int N, int K, int out_kind,
                                     void* out, int ldc, const float* gate, int gate_stride,
                                     const int* row_req, int splits);

/* Flash-style attention over packed segments: softmax(Q K^T / sqrt(dh)) V per segment and
 * head, no other mask.  q: dev bf16 rows [Nq][H*dh] with row stride ldq (elements); k likewise
 * [Nk] rows; vt: dev bf16 [H][dh][ldvt], the transposed values, segment s occupying columns
 * vt_off[s] .. vt_off[s]+len; cu_q / cu_k: host int32 [n_seg+1] prefix sums of query / key
 * rows per segment; vt_off: host int32 [n_seg], multiples of 64, each segment's columns
 * padded to a multiple of 64 with ZEROS (keys past the end are clamped copies whose
 * probabilities only cancel against zero values).  o: dev bf16 [Nq][ldo].  `work` is a dev
 * scratch of at least dit_op_attention_work_bytes(...) bytes.  q_prescaled != 0: the q rows
 * were multiplied by log2(e)/sqrt(dh) before rounding to bf16 (what the denoising step's q/k
 * norm writes; the result is the same function of the unscaled q).  logit_bound (only with
 * q_prescaled): if 0 < logit_bound <= 60 the caller guarantees |q.k| <= logit_bound for every
 * prescaled query and key, and the kernel keeps no running max; otherwise pass 0. */
size_t     dit_op_attention_work_bytes(int n_seg, const int* cu_q);
dit_status dit_op_attention(void* stream, const void* q, int ldq, const void* k, int ldk,
                            const void* vt, int ldvt, void* o, int ldo, int n_heads, int head_dim,
                            int n_seg, const int* cu_q, const int* cu_k, const int* vt_off,
                            void* work, size_t work_bytes, int q_prescaled, float logit_bound);

/* y = LN(x) * (1 + scale[row_req]) + shift[row_req], LN over the row without affine,
 * eps 1e-6.  x: dev float32 [M][d]; y: dev bf16 [M][d]; shift/scale: dev float32, row r at
 * shift + r*mod_stride; row_req: dev int32 [M] or NULL (all rows use request 0). */
dit_status dit_op_ln_modulate(void* stream, const float* x, void* y, int M, int d,
                              const float* shift, const float* scale, int mod_stride,
                              const int* row_req);

/* The denoising function Phi as an affine map: x <- a*x + b*v elementwise over n float32
 * elements (x, v dev). */
dit_status dit_op_latent_update(void* stream, float* x, const float* v, long long n, float a, float b);

#ifdef __cplusplus
}
#endif
#endif /* DIT_H */
