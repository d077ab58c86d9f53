/* C ABI of the Encode stage on one MI355X: a T5-v1.1-style text encoder that turns prompt
 * tokens into the condition c the Diffuse stage consumes (paper Section 2.1: the Encode stage
 * embeds the user guidance into a condition with a Transformer encoder; its pipeline table
 * names T5-XXL with 30-500 prompt tokens).  The paper does not describe the encoder's inside;
 * the published T5-v1.1 encoder is the reading taken:
 *
 *   x = E[token];  per layer:  h = RMSNorm(x) g1;  q,k,v = h Wq, h Wk, h Wv
 *                  x += softmax(q k^T + bias[head][bucket(key - query)]) v Wo     (no 1/sqrt(d))
 *                  h = RMSNorm(x) g2;  x += (gelu_tanh(h Wi0) * (h Wi1)) Wo2
 *   c = RMSNorm(x) g_final
 *   RMSNorm: x / sqrt(mean(x^2) + 1e-6), no mean subtraction; no biases; 32 relative-position
 *   buckets (16 per direction: distances 0..7 exact, then 8 + floor(8 ln(n/8)/ln 16), distances
 *   from 128 on share the last), one bias table [32][heads] for all layers.
 *
 * Conventions are those of dit.h (status codes, caller-owned device buffers, nothing
 * allocated by the library, errors kept per context, no CPU fallback).  Sequences are packed
 * back to back; a sequence attends only to itself.
 */
#ifndef DIT_ENCODER_H
#define DIT_ENCODER_H

#include "dit.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct enc_ctx enc_ctx;

typedef struct {
  int vocab;        /* rows of the embedding table                                      */
  int d_model;      /* multiple of 256                                                  */
  int n_heads;
  int head_dim;     /* 64 or 128; n_heads*head_dim a multiple of 256                    */
  int d_ff;         /* multiple of 256                                                  */
  int n_layers;
} enc_config;

enum { ENC_MAX_LEN = 1024 /* tokens per sequence */ };

/* Makes a context (no HIP call).  DIT_EINVAL / DIT_ESHAPE on a bad configuration. */
dit_status enc_create(const enc_config* cfg, int device, void* hip_stream, enc_ctx** out);
void       enc_destroy(enc_ctx* ctx);
const char* enc_last_error(const enc_ctx* ctx);

/* Bytes of the weight arena (matrices bf16 [out_pad][in_pad], embedding / bias tables and
 * gains fp32) and of the workspace for n_seq sequences of the given lengths (host int32
 * [n_seq], each 1..ENC_MAX_LEN; 0 is returned for an invalid list). */
size_t enc_weight_bytes(const enc_ctx* ctx);
size_t enc_workspace_bytes(const enc_ctx* ctx, int n_seq, const int* lens);
dit_status enc_bind(enc_ctx* ctx, void* dev_weights, size_t weight_bytes, void* dev_workspace,
                    size_t workspace_bytes);

/* Weights: matrices and tables ~ N(0, std^2) rounded to bf16 from the counter-based generator
 * of dit_init_weights (same key derivation from seed and tensor name), gains 1. */
dit_status enc_init_weights(enc_ctx* ctx, uint64_t seed, float std);
int        enc_tensor_count(const enc_ctx* ctx);
dit_status enc_tensor_info(const enc_ctx* ctx, int index, char* name, size_t name_len, int* rows_in,
                           int* cols_out, int* kind /* 0 matrix, 2 gain, 3 table */);
/* Host float32, logical layout [in][out] (tables [rows][cols], gains [n]); n = element count. */
dit_status enc_set_tensor(enc_ctx* ctx, const char* name, const float* host_src, size_t n);
dit_status enc_get_tensor(enc_ctx* ctx, const char* name, float* host_dst, size_t n);

/* Encodes n_seq packed sequences.  lens: host int32 [n_seq]; tokens: dev int32 [sum lens]
 * (ids outside [0, vocab) read row 0); out_bf16: dev bf16 [sum lens][d_model], the layout
 * dit_denoise_step / dit_sample take as `cond` for one request per sequence (may be NULL);
 * out_f32: dev float32 of the same shape (may be NULL).  Asynchronous on the context's stream. */
dit_status enc_forward(enc_ctx* ctx, int n_seq, const int* lens, const int* dev_tokens,
                       void* dev_out_bf16, float* dev_out_f32);

/* Capture points for tests, as dit_set_tap: "l<i>.ln1" (bf16), "l<i>.attn" (bf16),
 * "l<i>.x_attn" (fp32), "l<i>.act" (bf16), "l<i>.x_out" (fp32). */
dit_status enc_set_tap(enc_ctx* ctx, const char* point, void* dev_dst, size_t bytes);
void       enc_clear_taps(enc_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif
