/* C ABI of the Decode stage on one MI355X: an AutoencoderKL-style convolutional decoder that
 * maps the latent the Diffuse stage produced to pixels (paper Section 2.1: the latent result is
 * fed into the Decode stage, a memory-bound decoder; its batch-size figure names AutoEncoderKL).
 * The paper does not describe the decoder's inside; the published AutoencoderKL decoder is the
 * reading taken:
 *
 *   h = conv3x3(z);  mid: Res, h += proj(attention(GN(h))) (one head over all pixels), Res
 *   per level: n_res x Res (the first one changes the channel count), then, except after the
 *   last level, conv3x3(nearest 2x upsampling);  y = conv3x3(SiLU(GN(h)))
 *   Res(x) = shortcut(x) + conv3x3(SiLU(GN(conv3x3(SiLU(GN(x)))))), shortcut = 1x1 conv when the
 *   channel count changes; GN = GroupNorm(32 groups, eps 1e-6, affine); all convolutions have a
 *   bias and zero padding.
 *
 * Video form (temporal = 1), for the video models of the paper's pipeline table, whose latents
 * causal 3-D autoencoder decoders turn into frames; the paper does not describe them either.  The
 * reading taken keeps the structure above and changes what makes it a video decoder: every 3x3
 * convolution becomes a causal 3x3x3 convolution (output frame f reads frames f-2, f-1, f; frames
 * before the first are zero); 1x1 convolutions, GroupNorm and the mid-block attention act per
 * frame; at the first t_up level transitions the frame rate doubles before the spatial
 * upsampling, the first frame kept once and every later frame twice (F -> 2F - 1).
 *
 * Conventions are those of dit.h.
 */
#ifndef DIT_DECODER_H
#define DIT_DECODER_H

#include "dit.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dec_ctx dec_ctx;

enum { DEC_MAX_LEVELS = 6 };

typedef struct {
  int latent_ch;                  /* 1..64                                              */
  int out_ch;                     /* 1..4                                               */
  int n_levels;                   /* 1..DEC_MAX_LEVELS                                  */
  int channels[DEC_MAX_LEVELS];   /* width of each level, each in {64,128,256,512,1024} */
  int n_res;                      /* residual blocks per level, >= 1                    */
  int temporal;                   /* 0: image decoder; 1: causal video decoder          */
  int t_up;                       /* temporal = 1: level transitions that double the frame rate, 0..n_levels-1 (else 0) */
} dec_config;

dit_status dec_create(const dec_config* cfg, int device, void* hip_stream, dec_ctx** out);
void       dec_destroy(dec_ctx* ctx);
const char* dec_last_error(const dec_ctx* ctx);

/* A video decoder takes n = the latent frames of ONE video in every call below and produces
 * dec_frames_out(ctx, n) frames (an image decoder: n images; 0 for n < 1). */
int    dec_frames_out(const dec_ctx* ctx, int n);
/* Bytes of the weight arena and of the workspace for n latents of h x w.  0 for an invalid size:
 * h, w in 1..4096, (h*w) % 64 == 0 (whole k-slabs in the mid-block attention product) and
 * h*w <= 65536 (the score matrix is held whole); at most 128 images or output frames and,
 * with more than one, (h*w) % 256 == 0 (no group-norm chunk straddles images); fewer than 2^29
 * output pixels in all; one bordered image of the widest level (three of them for a video)
 * below 2^31 elements. */
size_t dec_weight_bytes(const dec_ctx* ctx);
size_t dec_workspace_bytes(const dec_ctx* ctx, int n, int h, int w);
dit_status dec_bind(dec_ctx* ctx, void* dev_weights, size_t weight_bytes, void* dev_workspace,
                    size_t workspace_bytes);

/* Weights ~ N(0, std^2) rounded to bf16 from the counter-based generator of dit_init_weights
 * (element index = row-major index in the logical [taps*C_in][C_out] matrix), biases 0, gains 1. */
dit_status dec_init_weights(dec_ctx* ctx, uint64_t seed, float std);
int        dec_tensor_count(const dec_ctx* ctx);
dit_status dec_tensor_info(const dec_ctx* ctx, int index, char* name, size_t name_len, int* rows_in,
                           int* cols_out, int* kind /* 0 matrix, 1 bias, 2 gain */);
/* Host float32; convolution weights as [taps*C_in][C_out], input index (3*ky + kx)*C_in + c; the
 * 3x3x3 convolutions of a video decoder: ((3*kf + ky)*3 + kx)*C_in + c, kf = 2 the output's own frame. */
dit_status dec_set_tensor(dec_ctx* ctx, const char* name, const float* host_src, size_t n);
dit_status dec_get_tensor(dec_ctx* ctx, const char* name, float* host_dst, size_t n);

/* Decodes a batch of n same-size latents (the paper batches the Decode stage like the others:
 * Appendix "Impact of Batch Size").  dev_latents: dev float32 [n][latent_ch][h][w] (per latent
 * the layout of the Diffuse stage's latents with one frame); dev_images: dev float32,
 * channels-last [n][h*2^(n_levels-1)][w*2^(n_levels-1)][out_ch].  Every image's result is
 * independent of its batch mates (statistics and attention are per image).  Video decoder:
 * dev_latents is one video, dev float32 [latent_ch][n][h][w] as the Diffuse stage leaves it, and
 * dev_images receives [dec_frames_out(ctx, n)] frames of that layout.  Asynchronous on the
 * context's stream. */
dit_status dec_forward(dec_ctx* ctx, int n, int h, int w, const float* dev_latents, float* dev_images);

/* Capture points for tests (fp32 channels-last [n * pixels][C]): "mid.res0", "mid.attn", "up<l>". */
dit_status dec_set_tap(dec_ctx* ctx, const char* point, void* dev_dst, size_t bytes);
void       dec_clear_taps(dec_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif
