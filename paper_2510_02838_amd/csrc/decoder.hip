// Row-wise kernels of the Decode stage (AutoencoderKL-style convolutional decoder).  Activations
// are channels-last; the residual stream is fp32 [pixels][C]; inputs of 3x3 convolutions are
// bf16 images with a one-pixel zero border, [(H+2)*(W+2)][C], so that the convolution is a
// matrix product with shifted row addresses (gemm.hip) and needs no masking.  A batch of B
// same-size images is B such streams / bordered images back to back.
#include "dit_internal.h"

namespace dit {

namespace {
__device__ __forceinline__ uint16_t d_f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ uint32_t d_pack2(float a, float b) { return (uint32_t)d_f2bf(a) | ((uint32_t)d_f2bf(b) << 16); }
__device__ __forceinline__ float d_silu(float x) { return x * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x)); }
// destination row of pixel (y, x): bordered image of width W if pad, plain otherwise
__device__ __forceinline__ long long dst_pixel(int y, int x, int W, int pad) {
  return pad ? (long long)(y + 1) * (W + 2) + (x + 1) : (long long)y * W + x;
}
}  // namespace

// latents fp32 channels-first [B][C][H][W] -> bf16 bordered channels-last [B][(H+2)(W+2)][Cpad],
// channels from C on are zero (the border is zero from a fill of the whole buffer by the caller)
__global__ __launch_bounds__(256) void latent_to_image_kernel(const float* __restrict__ z, bf16_t* __restrict__ out,
                                                              int C, int H, int W, int Cpad, int B, int frames) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long per = (long long)H * W * C;
  if (i >= per * B) return;
  const int b = (int)(i / per);
  const long long r = i - b * per;
  const int c = (int)(r % C);
  const long long p = r / C;
  const int y = (int)(p / W), x = (int)(p % W);
  out[((long long)b * (H + 2) * (W + 2) + dst_pixel(y, x, W, 1)) * Cpad + c] = d_f2bf(z[(frames ? ((long long)c * frames + b) : ((long long)b * C + c)) * H * W + (long long)y * W + x]);
}

void launch_latent_to_image(hipStream_t s, const float* z, bf16_t* out, int C, int H, int W, int Cpad, int B, int frames) {
  const long long n = (long long)B * H * W * C;
  if (n) hipLaunchKernelGGL(latent_to_image_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, z, out, C, H, W, Cpad, B, frames);
}

// zero border of a bordered image [(H+2)(W+2)][C]: rows 0 and H+1, columns 0 and W+1
__global__ __launch_bounds__(256) void zero_border_kernel(bf16_t* __restrict__ img, int H, int W, int C) {
  img += (size_t)blockIdx.y * (H + 2) * (W + 2) * C;       // one bordered image per blockIdx.y
  const int o8 = C >> 3;                                   // 16-byte pieces per pixel
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long nb = 2LL * (W + 2) + 2LL * H;            // border pixels
  if (i >= nb * o8) return;
  const long long b = i / o8;
  const int c = (int)(i % o8) * 8;
  long long pix;
  if (b < W + 2) pix = b;                                                   // top row
  else if (b < 2LL * (W + 2)) pix = (long long)(H + 1) * (W + 2) + (b - (W + 2));   // bottom row
  else { const long long r = b - 2LL * (W + 2); pix = (r / 2 + 1) * (W + 2) + ((r & 1) ? W + 1 : 0); }
  *(uint4*)(img + pix * C + c) = make_uint4(0, 0, 0, 0);
}
void launch_zero_border(hipStream_t s, bf16_t* img, int H, int W, int C, int B) {
  const long long n = (2LL * (W + 2) + 2LL * H) * (C / 8);
  if (n && B) hipLaunchKernelGGL(zero_border_kernel, dim3((unsigned)((n + 255) / 256), B), dim3(256), 0, s, img, H, W, C);
}

// ---- group norm ---------------------------------------------------------------------------
// pass 1: per chunk of GN_CHUNK pixels, per channel: sum and sum of squares.  A thread owns 4
// consecutive channels and strides over the chunk's pixels; threads that share channels combine
// through LDS in a fixed order.  partial: [chunks][C][2].  C is a power of two in 64..1024.
constexpr int GN_CHUNK = 256;
__global__ __launch_bounds__(256) void gn_partial_kernel(const float* __restrict__ x, float* __restrict__ partial,
                                                         long long P, int C, int qsh) {
  extern __shared__ float red[];                // [pix_par][C][2]
  const int qpc = C >> 2;                       // channel quads per pixel = 1 << qsh
  const int tid = threadIdx.x;
  const int quad = tid & (qpc - 1), lane_pix = tid >> qsh, pix_par = 256 >> qsh;
  const long long p0 = (long long)blockIdx.x * GN_CHUNK;
  float s[4] = {0, 0, 0, 0}, q[4] = {0, 0, 0, 0};
  const float4* xp = (const float4*)(x + p0 * C) + quad;
  if (p0 + GN_CHUNK <= P) {
    // whole chunk: four independent loads in flight per thread
    for (int pp = lane_pix; pp < GN_CHUNK; pp += 4 * pix_par) {
      float4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = xp[(size_t)(pp + u * pix_par) * qpc];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        s[0] += v[u].x; s[1] += v[u].y; s[2] += v[u].z; s[3] += v[u].w;
        q[0] += v[u].x * v[u].x; q[1] += v[u].y * v[u].y; q[2] += v[u].z * v[u].z; q[3] += v[u].w * v[u].w;
      }
    }
  } else {
    for (int pp = lane_pix; pp < GN_CHUNK && p0 + pp < P; pp += pix_par) {
      const float4 v = xp[(size_t)pp * qpc];
      s[0] += v.x; s[1] += v.y; s[2] += v.z; s[3] += v.w;
      q[0] += v.x * v.x; q[1] += v.y * v.y; q[2] += v.z * v.z; q[3] += v.w * v.w;
    }
  }
  {
    float* r = red + ((size_t)lane_pix * C + quad * 4) * 2;
#pragma unroll
    for (int j = 0; j < 4; ++j) { r[2 * j] = s[j]; r[2 * j + 1] = q[j]; }
  }
  __syncthreads();
  for (int c = tid; c < C; c += 256) {
    float a = 0.f, b = 0.f;
    for (int l = 0; l < pix_par; ++l) { a += red[((size_t)l * C + c) * 2]; b += red[((size_t)l * C + c) * 2 + 1]; }
    partial[((size_t)blockIdx.x * C + c) * 2] = a;
    partial[((size_t)blockIdx.x * C + c) * 2 + 1] = b;
  }
}
// pass 2: one workgroup per (group, share of the chunks): chunk sums of the group's channels added
// in fixed order in float64.  With one share per group the workgroup writes stats[g] = (mean,
// 1/sqrt(var + eps)) itself; with several it leaves (sum, sum of squares) in part[g][share] for
// gn_combine_kernel (many chunks: 32 workgroups alone would take longer than the apply pass).
__global__ __launch_bounds__(256) void gn_finalize_kernel(const float* __restrict__ partial, float2* __restrict__ stats,
                                                          double2* __restrict__ part, int chunks, int C, int groups, long long P) {
  __shared__ double rs[256], rq[256];
  const int g = blockIdx.x, cpg = C / groups, tid = threadIdx.x;
  const int shares = gridDim.y, sh = blockIdx.y;
  const int img = blockIdx.z;                    // chunks, P: per image; an image's chunks are consecutive
  partial += (size_t)img * chunks * C * 2;
  stats += img * groups;
  part += img * groups * shares;
  const int c0 = (int)((long long)chunks * sh / shares), c1 = (int)((long long)chunks * (sh + 1) / shares);
  double a = 0.0, b = 0.0;
  for (int ch = c0 + tid; ch < c1; ch += 256)
    for (int c = 0; c < cpg; ++c) {
      const float* pp = partial + ((size_t)ch * C + g * cpg + c) * 2;
      a += (double)pp[0]; b += (double)pp[1];
    }
  rs[tid] = a; rq[tid] = b;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (tid < o) { rs[tid] += rs[tid + o]; rq[tid] += rq[tid + o]; }
    __syncthreads();
  }
  if (tid == 0) {
    if (shares > 1) { part[g * shares + sh] = make_double2(rs[0], rq[0]); return; }
    const double n = (double)P * cpg, mean = rs[0] / n;
    double var = rq[0] / n - mean * mean;
    if (var < 0.0) var = 0.0;
    stats[g] = make_float2((float)mean, (float)(1.0 / sqrt(var + 1e-6)));
  }
}
__global__ __launch_bounds__(64) void gn_combine_kernel(const double2* __restrict__ part, float2* __restrict__ stats,
                                                        int shares, int cpg, int groups, long long P) {
  const int g = threadIdx.x;
  if (g >= groups) return;
  part += blockIdx.x * groups * shares;          // one image per workgroup
  stats += blockIdx.x * groups;
  double a = 0.0, b = 0.0;
  for (int s = 0; s < shares; ++s) { a += part[g * shares + s].x; b += part[g * shares + s].y; }
  const double n = (double)P * cpg, mean = a / n;
  double var = b / n - mean * mean;
  if (var < 0.0) var = 0.0;
  stats[g] = make_float2((float)mean, (float)(1.0 / sqrt(var + 1e-6)));
}
// pass 3: y = (x - mean_g) rstd_g gamma_c + beta_c, optional SiLU, bf16, bordered or plain rows.
// One image row per blockIdx.y; a thread takes 8 consecutive channels of four consecutive pixels (gain, bias and
// the group statistics are fetched once for the four, and the four pixels' loads are in flight together).
__global__ __launch_bounds__(256) void gn_apply_kernel(const float* __restrict__ x, const float2* __restrict__ stats,
                                                       const float* __restrict__ gamma, const float* __restrict__ beta,
                                                       bf16_t* __restrict__ out, int W, int C, int osh, int gsh,
                                                       int silu, int pad, int groups) {
  const int i = blockIdx.x * 256 + threadIdx.x;      // unit: 8 channels of a group of four pixels of the row
  const int opc = C >> 3;                            // = 1 << osh
  if (i >= ((W + 3) >> 2) * opc) return;
  const int H = gridDim.y, img = blockIdx.z;         // one image per blockIdx.z
  x += (size_t)img * H * W * C;
  out += (size_t)img * (pad ? (size_t)(H + 2) * (W + 2) : (size_t)H * W) * C;
  stats += img * groups;
  const int y = blockIdx.y, x0 = (i >> osh) * 4, c = (i & (opc - 1)) * 8;
  const float* xr = x + ((size_t)y * W + x0) * C + c;
  float4 v0[4], v1[4];
#pragma unroll
  for (int k = 0; k < 4; ++k)
    if (x0 + k < W) { v0[k] = *(const float4*)(xr + (size_t)k * C); v1[k] = *(const float4*)(xr + (size_t)k * C + 4); }
  const float4 g0 = *(const float4*)(gamma + c), g1 = *(const float4*)(gamma + c + 4);
  const float4 b0 = *(const float4*)(beta + c), b1 = *(const float4*)(beta + c + 4);
  const float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
  const float bb[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
  float sc[8], sh[8];                                // y = x * sc + sh
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float2 st = stats[(c + j) >> gsh];
    sc[j] = st.y * gg[j];
    sh[j] = bb[j] - st.x * sc[j];
  }
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    if (x0 + k >= W) break;
    float r[8] = {v0[k].x, v0[k].y, v0[k].z, v0[k].w, v1[k].x, v1[k].y, v1[k].z, v1[k].w};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      r[j] = r[j] * sc[j] + sh[j];
      if (silu) r[j] = d_silu(r[j]);
    }
    uint4 w;
    w.x = d_pack2(r[0], r[1]); w.y = d_pack2(r[2], r[3]); w.z = d_pack2(r[4], r[5]); w.w = d_pack2(r[6], r[7]);
    *(uint4*)(out + dst_pixel(y, x0 + k, W, pad) * C + c) = w;
  }
}

// B images of H x W; statistics per image and group.  ready_chunks > 0: `partial` already holds
// that many per-chunk channel sums PER IMAGE (written by the epilogue of the convolution that
// produced x; chunks do not straddle images): pass 1 is skipped.  With B > 1 the standalone
// pass 1 needs H*W to be a multiple of its chunk (256 pixels).
void launch_group_norm(hipStream_t s, const float* x, const float* gamma, const float* beta, bf16_t* out,
                       float* partial, float2* stats, int H, int W, int C, int groups, int silu, int pad,
                       int ready_chunks, int B) {
  const long long P = (long long)H * W;
  if (P == 0 || B == 0) return;
  int chunks = ready_chunks;
  int csh = 0;
  while ((1 << csh) < C) ++csh;                  // C = 1 << csh
  int gsh = 0;
  while ((groups << gsh) < C) ++gsh;             // channels per group = 1 << gsh
  if (chunks <= 0) {
    chunks = (int)((P + GN_CHUNK - 1) / GN_CHUNK);
    const int pix_par = 256 >> (csh - 2);
    hipLaunchKernelGGL(gn_partial_kernel, dim3(chunks * B), dim3(256), (size_t)pix_par * C * 2 * sizeof(float), s, x, partial, P * B, C, csh - 2);
  }
  // stats: [B][groups] float2, then (GN_STATS_HEAD bytes on) the [B][groups][shares] float64 pairs of the two-stage form
  const int shares = chunks >= 4096 ? 16 : (chunks >= 1024 ? 4 : 1);
  double2* part = (double2*)((unsigned char*)stats + GN_STATS_HEAD);
  hipLaunchKernelGGL(gn_finalize_kernel, dim3(groups, shares, B), dim3(256), 0, s, partial, stats, part, chunks, C, groups, P);
  if (shares > 1) hipLaunchKernelGGL(gn_combine_kernel, dim3(B), dim3(64), 0, s, part, stats, shares, C / groups, groups, P);
  const int units = ((W + 3) >> 2) * (C >> 3);
  hipLaunchKernelGGL(gn_apply_kernel, dim3((units + 255) / 256, H, B), dim3(256), 0, s, x, stats, gamma, beta, out, W, C, csh - 3, gsh, silu, pad, groups);
}
size_t group_norm_partial_bytes(long long pixels, int C) {
  return (size_t)((pixels + GN_CHUNK - 1) / GN_CHUNK) * C * 2 * sizeof(float);
}

// nearest 2x upsampling of the fp32 stream into a bf16 bordered image: out pixel (y, x) = in (y/2, x/2).
// A thread reads 8 channels of one input pixel once and writes the four output pixels that show it.
__global__ __launch_bounds__(256) void upsample_pad_kernel(const float* __restrict__ x, bf16_t* __restrict__ out,
                                                           int H, int W, int C, int frame_up) {       // H, W: input size
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  const int opc = C >> 3;
  const int W2 = 2 * W;
  if (i >= (long long)H * W * opc) return;
  x += (size_t)(frame_up ? (blockIdx.y + 1) >> 1 : blockIdx.y) * H * W * C;     // one output image per blockIdx.y
  out += (size_t)blockIdx.y * (2 * H + 2) * (W2 + 2) * C;
  const long long p = i / opc;
  const int c = (int)(i % opc) * 8;
  const int y = (int)(p / W), xx = (int)(p % W);
  const float4* src = (const float4*)(x + p * C + c);
  const float4 v0 = src[0], v1 = src[1];
  uint4 w;
  w.x = d_pack2(v0.x, v0.y); w.y = d_pack2(v0.z, v0.w); w.z = d_pack2(v1.x, v1.y); w.w = d_pack2(v1.z, v1.w);
#pragma unroll
  for (int dy = 0; dy < 2; ++dy)
#pragma unroll
    for (int dx = 0; dx < 2; ++dx)
      *(uint4*)(out + dst_pixel(2 * y + dy, 2 * xx + dx, W2, 1) * C + c) = w;
}
void launch_upsample_pad(hipStream_t s, const float* x, bf16_t* out, int H, int W, int C, int B, int frame_up) {
  const long long n = (long long)H * W * (C / 8);
  if (n && B) hipLaunchKernelGGL(upsample_pad_kernel, dim3((unsigned)((n + 255) / 256), B), dim3(256), 0, s, x, out, H, W, C, frame_up);
}

// fp32 -> bf16, 4 elements per thread (plain rows)
// (a workgroup takes 4 x 256 float4s, a thread one of each quarter: four loads in flight per thread)
__global__ __launch_bounds__(256) void cast_bf16_kernel(const float* __restrict__ x, bf16_t* __restrict__ out, long long n4) {
  const long long i0 = (long long)blockIdx.x * 1024 + threadIdx.x;
  float4 v[4];
#pragma unroll
  for (int k = 0; k < 4; ++k)
    if (i0 + k * 256 < n4) v[k] = ((const float4*)x)[i0 + k * 256];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    if (i0 + k * 256 >= n4) break;
    uint2 w;
    w.x = d_pack2(v[k].x, v[k].y); w.y = d_pack2(v[k].z, v[k].w);
    ((uint2*)out)[i0 + k * 256] = w;
  }
}
void launch_cast_bf16(hipStream_t s, const float* x, bf16_t* out, long long n) {
  if (n) hipLaunchKernelGGL(cast_bf16_kernel, dim3((unsigned)((n / 4 + 1023) / 1024)), dim3(256), 0, s, x, out, n / 4);
}

// row softmax of fp32 scores times `scale`, written as bf16 with row stride ldo; columns from n to
// ldo are written as zeros.  One workgroup per row, three passes over the row (max, sum, write).
__global__ __launch_bounds__(256) void softmax_rows_kernel(const float* __restrict__ sc, int lds_, bf16_t* __restrict__ out,
                                                           int ldo, int n, float scale_log2) {
  __shared__ float red[256];
  const float* r = sc + (size_t)blockIdx.x * lds_;
  const int tid = threadIdx.x;
  float m = -INFINITY;
  for (int j = tid; j < n; j += 256) m = fmaxf(m, r[j]);
  red[tid] = m; __syncthreads();
  for (int o = 128; o > 0; o >>= 1) { if (tid < o) red[tid] = fmaxf(red[tid], red[tid + o]); __syncthreads(); }
  m = red[0]; __syncthreads();
  float s = 0.f;
  for (int j = tid; j < n; j += 256) s += __builtin_amdgcn_exp2f((r[j] - m) * scale_log2);
  red[tid] = s; __syncthreads();
  for (int o = 128; o > 0; o >>= 1) { if (tid < o) red[tid] += red[tid + o]; __syncthreads(); }
  const float inv = 1.0f / red[0];
  bf16_t* o_ = out + (size_t)blockIdx.x * ldo;
  for (int j = tid; j < ldo; j += 256)
    o_[j] = j < n ? d_f2bf(__builtin_amdgcn_exp2f((r[j] - m) * scale_log2) * inv) : (bf16_t)0;
}
// the same with the row held in registers between the passes (n <= 256 * 4 * NV, n % 4 == 0,
// ldo % 4 == 0): one read of the scores instead of three
template <int NV>
__global__ __launch_bounds__(256) void softmax_rows_reg_kernel(const float* __restrict__ sc, int lds_, bf16_t* __restrict__ out,
                                                               int ldo, int n, float scale_log2) {
  __shared__ float red[4];
  const float4* r = (const float4*)(sc + (size_t)blockIdx.x * lds_);
  const int tid = threadIdx.x, n4 = n >> 2;
  float4 v[NV];
  float m = -INFINITY;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int j = i * 256 + tid;
    v[i] = j < n4 ? r[j] : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
    m = fmaxf(fmaxf(m, fmaxf(v[i].x, v[i].y)), fmaxf(v[i].z, v[i].w));
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
  if ((tid & 63) == 0) red[tid >> 6] = m;
  __syncthreads();
  m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    v[i].x = __builtin_amdgcn_exp2f((v[i].x - m) * scale_log2); v[i].y = __builtin_amdgcn_exp2f((v[i].y - m) * scale_log2);
    v[i].z = __builtin_amdgcn_exp2f((v[i].z - m) * scale_log2); v[i].w = __builtin_amdgcn_exp2f((v[i].w - m) * scale_log2);
    s += (v[i].x + v[i].y) + (v[i].z + v[i].w);          // (exp2(-inf) = 0 past the row's end)
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
  if ((tid & 63) == 0) red[tid >> 6] = s;
  __syncthreads();
  const float inv = 1.0f / ((red[0] + red[1]) + (red[2] + red[3]));
  uint2* o_ = (uint2*)(out + (size_t)blockIdx.x * ldo);
  const int o4 = ldo >> 2;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int j = i * 256 + tid;
    if (j < o4) {
      uint2 w;
      w.x = d_pack2(v[i].x * inv, v[i].y * inv); w.y = d_pack2(v[i].z * inv, v[i].w * inv);
      o_[j] = w;                                         // zeros from n to ldo
    }
  }
}
void launch_softmax_rows(hipStream_t s, const float* sc, int lds_, bf16_t* out, int ldo, int rows, int n, float scale_log2) {
  if (!rows) return;
  const bool vec = n % 4 == 0 && ldo % 4 == 0 && lds_ % 4 == 0 && ldo <= 16384 && n <= ldo;
  if (vec && ldo <= 4096) hipLaunchKernelGGL(softmax_rows_reg_kernel<4>, dim3(rows), dim3(256), 0, s, sc, lds_, out, ldo, n, scale_log2);
  else if (vec) hipLaunchKernelGGL(softmax_rows_reg_kernel<16>, dim3(rows), dim3(256), 0, s, sc, lds_, out, ldo, n, scale_log2);
  else hipLaunchKernelGGL(softmax_rows_kernel, dim3(rows), dim3(256), 0, s, sc, lds_, out, ldo, n, scale_log2);
}

// 3x3 convolution to a few output channels (the decoder's last layer: 3), read-bound: a product
// on the matrix cores would compute 128-column tiles for 3 columns.  C/8 lanes share a pixel, a
// lane owns 8 channels: its 9 x OC weight pieces stay in registers while the wave walks over
// pixels (coalesced 16-byte loads of whole pixel rows), bf16 pair dot products accumulate in
// fp32 and the lanes of a pixel are summed by shuffles.  img: bordered bf16 image
// [(H+2)(W+2)][C]; w: bf16 [>= OC][ldw], input index (3 ky + kx) C + c; out: fp32 [H W][OC].
// C in {64, 128, 256, 512}.
template <int OC>
__global__ __launch_bounds__(256) void conv3_small_kernel(const bf16_t* __restrict__ img, const bf16_t* __restrict__ w, int ldw,
                                                          const float* __restrict__ bias, float* __restrict__ out,
                                                          int H, int W, int C, int lsh, int B, int accumulate) {
  typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
  const int lane = threadIdx.x & 63;
  const int lpp = 1 << lsh;                         // lanes per pixel = C / 8
  const int sub = lane & (lpp - 1), pl = lane >> lsh, ppw = 64 >> lsh;
  uint4 wr[9][OC];
#pragma unroll
  for (int tap = 0; tap < 9; ++tap)
#pragma unroll
    for (int o = 0; o < OC; ++o) wr[tap][o] = *(const uint4*)(w + (size_t)o * ldw + tap * C + sub * 8);
  const long long PI = (long long)H * W, P = PI * B;      // B images back to back
  const long long wave = (long long)blockIdx.x * 4 + (threadIdx.x >> 6), nwaves = (long long)gridDim.x * 4;
  for (long long p0 = wave * ppw; p0 < P; p0 += nwaves * ppw) {
    const long long p = p0 + pl;
    const bool ok = p < P;
    const long long pc = ok ? p : P - 1;
    const int bimg = (int)(pc / PI);
    const long long pr = pc - bimg * PI;
    const int y = (int)(pr / W) + bimg * (H + 2), x = (int)(pr % W);   // row in the stack of bordered images
    float acc[OC];
#pragma unroll
    for (int o = 0; o < OC; ++o) acc[o] = 0.f;
    uint4 v[9];
#pragma unroll
    for (int tap = 0; tap < 9; ++tap)
      v[tap] = *(const uint4*)(img + ((size_t)(y + tap / 3) * (W + 2) + (x + tap % 3)) * C + sub * 8);
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
      const uint32_t vv[4] = {v[tap].x, v[tap].y, v[tap].z, v[tap].w};
#pragma unroll
      for (int o = 0; o < OC; ++o) {
        const uint32_t wv[4] = {wr[tap][o].x, wr[tap][o].y, wr[tap][o].z, wr[tap][o].w};
#pragma unroll
        for (int q = 0; q < 4; ++q)
          acc[o] = __builtin_amdgcn_fdot2_f32_bf16(*(const bf2*)&vv[q], *(const bf2*)&wv[q], acc[o], false);
      }
    }
    for (int off = 1; off < lpp; off <<= 1)
#pragma unroll
      for (int o = 0; o < OC; ++o) acc[o] += __shfl_xor(acc[o], off);
    if (ok && sub == 0) {
#pragma unroll
      for (int o = 0; o < OC; ++o) out[p * OC + o] = (accumulate ? out[p * OC + o] : 0.f) + acc[o] + (bias ? bias[o] : 0.f);
    }
  }
}
bool launch_conv3_small(hipStream_t s, const bf16_t* img, const bf16_t* w, int ldw, const float* bias, float* out,
                        int H, int W, int C, int OC, int B, int accumulate) {
  if (OC < 1 || OC > 4 || (C != 64 && C != 128 && C != 256 && C != 512)) return false;
  const long long P = (long long)H * W * B;
  if (P == 0) return true;
  int lsh = 0;
  while ((8 << lsh) < C) ++lsh;
  const long long groups = (P + (64 >> lsh) - 1) / (64 >> lsh);       // wave-loads of pixels
  const long long want = (groups + 3) / 4;
  dim3 g((unsigned)(want < 4096 ? want : 4096)), b(256);
  switch (OC) {
    case 1: hipLaunchKernelGGL(conv3_small_kernel<1>, g, b, 0, s, img, w, ldw, bias, out, H, W, C, lsh, B, accumulate); break;
    case 2: hipLaunchKernelGGL(conv3_small_kernel<2>, g, b, 0, s, img, w, ldw, bias, out, H, W, C, lsh, B, accumulate); break;
    case 3: hipLaunchKernelGGL(conv3_small_kernel<3>, g, b, 0, s, img, w, ldw, bias, out, H, W, C, lsh, B, accumulate); break;
    default: hipLaunchKernelGGL(conv3_small_kernel<4>, g, b, 0, s, img, w, ldw, bias, out, H, W, C, lsh, B, accumulate); break;
  }
  return true;
}

// out[(y*W + x)*C + c] (fp32, channels-last, C small) from the fp32 product rows: plain copy is
// not needed; the last convolution writes fp32 rows [pixels][ldc] and this kernel compacts them
__global__ __launch_bounds__(256) void compact_rows_kernel(const float* __restrict__ src, int lds_, float* __restrict__ dst,
                                                           long long P, int C) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= P * C) return;
  dst[i] = src[(i / C) * lds_ + (i % C)];
}
void launch_compact_rows(hipStream_t s, const float* src, int lds_, float* dst, long long P, int C) {
  if (P) hipLaunchKernelGGL(compact_rows_kernel, dim3((unsigned)((P * C + 255) / 256)), dim3(256), 0, s, src, lds_, dst, P, C);
}

}  // namespace dit
