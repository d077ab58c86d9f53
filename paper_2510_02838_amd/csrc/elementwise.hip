// HBM-bound kernels of the denoising step: adaLN layer norm + modulation, per-head q/k RMS
// norm + rotary code, V transpose, patchify / unpatchify + latent update, the small-M
// matrix-vector products of the conditioning path, and weight initialisation.
// All of them are coalesced row-wise kernels with wavefront (64-lane) reductions.
#include "dit_internal.h"

namespace dit {

__device__ __forceinline__ uint16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf2f(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ uint32_t pack2(float a, float b) { return (uint32_t)f2bf(a) | ((uint32_t)f2bf(b) << 16); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// ---------------------------------------------------------------------------------------
// adaLN:  y = LN(x) * (1 + scale[req]) + shift[req]        (or LN(x) * gain + beta)
// one wave per row; the row lives in registers between the two passes (mean, variance).
// ---------------------------------------------------------------------------------------
template <int MAXV>
__global__ __launch_bounds__(256) void ln_modulate_kernel(const float* __restrict__ x, bf16_t* __restrict__ y,
                                                          int M, int d, const float* __restrict__ shift,
                                                          const float* __restrict__ scale, int mod_stride,
                                                          const int* __restrict__ row_req,
                                                          const float* __restrict__ gain,
                                                          const float* __restrict__ beta,
                                                          bf16_t* __restrict__ y_lo, int split,
                                                          const float* __restrict__ shift2,
                                                          const float* __restrict__ scale2) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= M) return;
  const int lane = threadIdx.x & 63;
  const int nv = d >> 8;                       // float4 vectors per lane
  const float4* xr = (const float4*)(x + (size_t)row * d);
  // The modulation vectors do not depend on the row's statistics: their loads go out with the row's own, ahead
  // of the two reductions, instead of behind them.
  const float4 *sh, *sc;
  bool plus_one;
  if (gain) {
    sc = (const float4*)gain; sh = (const float4*)beta; plus_one = false;
  } else {
    const size_t mo = (size_t)(row_req ? row_req[row] : 0) * mod_stride;
    const bool second = row >= split;     // rows from `split` on take the second stream's vectors
    sc = (const float4*)((second ? scale2 : scale) + mo); sh = (const float4*)((second ? shift2 : shift) + mo);
    plus_one = true;
  }
  constexpr bool PRE = MAXV <= 12;        // (wider rows have no registers for it: there the loads stay behind)
  float4 v[MAXV], ma[PRE ? MAXV : 1], mb[PRE ? MAXV : 1];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < MAXV; ++i)
    if (i < nv) v[i] = xr[i * 64 + lane];
  if constexpr (PRE) {
#pragma unroll
    for (int i = 0; i < MAXV; ++i)
      if (i < nv) { ma[i] = sc[i * 64 + lane]; mb[i] = sh[i * 64 + lane]; }
  }
#pragma unroll
  for (int i = 0; i < MAXV; ++i)
    if (i < nv) s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
  const float mean = wave_sum(s) / (float)d;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < MAXV; ++i)
    if (i < nv) {
      v[i].x -= mean; v[i].y -= mean; v[i].z -= mean; v[i].w -= mean;
      q += (v[i].x * v[i].x + v[i].y * v[i].y) + (v[i].z * v[i].z + v[i].w * v[i].w);
    }
  const float rstd = rsqrtf(wave_sum(q) / (float)d + 1e-6f);
  uint2* yr = (uint2*)(y + (size_t)row * d);
#pragma unroll
  for (int i = 0; i < MAXV; ++i)
    if (i < nv) {
      float4 a, b;
      if constexpr (PRE) { a = ma[i]; b = mb[i]; } else { a = sc[i * 64 + lane]; b = sh[i * 64 + lane]; }
      if (plus_one) { a.x += 1.f; a.y += 1.f; a.z += 1.f; a.w += 1.f; }
      const float r0 = v[i].x * rstd * a.x + b.x, r1 = v[i].y * rstd * a.y + b.y;
      const float r2 = v[i].z * rstd * a.z + b.z, r3 = v[i].w * rstd * a.w + b.w;
      uint2 w;
      w.x = pack2(r0, r1);
      w.y = pack2(r2, r3);
      yr[i * 64 + lane] = w;
      if (y_lo) {   // second bf16 term: value = hi + lo to about 16 mantissa bits
        uint2 l;
        l.x = pack2(r0 - bf2f((uint16_t)(w.x & 0xFFFF)), r1 - bf2f((uint16_t)(w.x >> 16)));
        l.y = pack2(r2 - bf2f((uint16_t)(w.y & 0xFFFF)), r3 - bf2f((uint16_t)(w.y >> 16)));
        ((uint2*)(y_lo + (size_t)row * d))[i * 64 + lane] = l;
      }
    }
}

void launch_ln_modulate(hipStream_t s, const float* x, bf16_t* y, int M, int d, const float* shift,
                        const float* scale, int mod_stride, const int* row_req, const float* gain,
                        const float* beta, bf16_t* y_lo, int split, const float* shift2, const float* scale2) {
  if (split < 0 || !shift2) { split = M; shift2 = shift; scale2 = scale; }
  if (M == 0) return;
  dim3 g((M + 3) / 4), b(256);
  if (d <= 1024) hipLaunchKernelGGL(ln_modulate_kernel<4>, g, b, 0, s, x, y, M, d, shift, scale, mod_stride, row_req, gain, beta, y_lo, split, shift2, scale2);
  else if (d <= 1536) hipLaunchKernelGGL(ln_modulate_kernel<6>, g, b, 0, s, x, y, M, d, shift, scale, mod_stride, row_req, gain, beta, y_lo, split, shift2, scale2);
  else if (d <= 3072) hipLaunchKernelGGL(ln_modulate_kernel<12>, g, b, 0, s, x, y, M, d, shift, scale, mod_stride, row_req, gain, beta, y_lo, split, shift2, scale2);
  else hipLaunchKernelGGL(ln_modulate_kernel<20>, g, b, 0, s, x, y, M, d, shift, scale, mod_stride, row_req, gain, beta, y_lo, split, shift2, scale2);
}

// ---------------------------------------------------------------------------------------
// q/k per-head RMS norm (+ rotary code).  A lane owns 8 consecutive elements (16 bytes) of one
// head of one row; the dh/8 lanes of a head reduce with shuffles.
// ---------------------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256) void qknorm_rope_kernel(const bf16_t* __restrict__ qkv, int ld, int M, int d,
                                                          const float* __restrict__ qgain,
                                                          const float* __restrict__ kgain,
                                                          const float2* __restrict__ rope,
                                                          const int* __restrict__ dst_row,
                                                          bf16_t* __restrict__ qo, bf16_t* __restrict__ ko,
                                                          int ldo, int k_col_off, int do_k, int split,
                                                          const float* __restrict__ qgain2,
                                                          const float* __restrict__ kgain2, float qscale) {
  const int cpr = d >> 3;                                // 16-byte chunks per row
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  const bool ok = idx < (long long)M * cpr;              // (heads never straddle the tail: cpr % (DH/8) == 0)
  const int row = ok ? (int)(idx / cpr) : M - 1;
  const int col = ok ? (int)(idx % cpr) * 8 : 0;
  if (row >= split) { qgain = qgain2; kgain = kgain2; }   // second stream's gains
  const int hc = col % DH;                               // first element within the head
  const int drow = dst_row ? dst_row[row] : row;
  float2 cs[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) cs[p] = make_float2(1.f, 0.f);
  if (rope) {
    const float4* rp = (const float4*)(rope + (size_t)drow * (DH / 2) + (hc >> 1));
    const float4 r0 = rp[0], r1 = rp[1];
    cs[0] = make_float2(r0.x, r0.y); cs[1] = make_float2(r0.z, r0.w);
    cs[2] = make_float2(r1.x, r1.y); cs[3] = make_float2(r1.z, r1.w);
  }
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    if (which == 1 && !do_k) break;
    const uint4 raw = *(const uint4*)(qkv + (size_t)row * ld + (which ? k_col_off : 0) + col);
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
    float x[8];
    float ss = 0.f;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      x[2 * p] = bf2f((uint16_t)(w[p] & 0xFFFF));
      x[2 * p + 1] = bf2f((uint16_t)(w[p] >> 16));
      ss += x[2 * p] * x[2 * p] + x[2 * p + 1] * x[2 * p + 1];
    }
#pragma unroll
    for (int o = DH / 16; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    const float r = rsqrtf(ss / (float)DH + 1e-6f) * (which ? 1.f : qscale);
    const float4* gp = (const float4*)((which ? kgain : qgain) + hc);
    const float4 g0 = gp[0], g1 = gp[1];
    const float g[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
    uint4 out;
    uint32_t* ow = (uint32_t*)&out;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const float a = x[2 * p] * r * g[2 * p], b = x[2 * p + 1] * r * g[2 * p + 1];
      ow[p] = pack2(a * cs[p].x - b * cs[p].y, a * cs[p].y + b * cs[p].x);
    }
    if (ok) *(uint4*)((which ? ko : qo) + (size_t)drow * ldo + col) = out;
  }
}

void launch_qknorm_rope(hipStream_t s, const bf16_t* qkv, int ld, int M, int H, int dh, const float* qgain,
                        const float* kgain, const float2* rope, const int* dst_row, bf16_t* qo, bf16_t* ko,
                        int ldo, int k_col_off, int do_k, int split, const float* qgain2, const float* kgain2,
                        float qscale) {
  if (M == 0) return;
  if (split < 0 || !qgain2) { split = M; qgain2 = qgain; kgain2 = kgain; }
  const int d = H * dh;
  const long long total = (long long)M * (d / 8);
  dim3 g((unsigned)((total + 255) / 256)), b(256);
  if (dh == 64) hipLaunchKernelGGL(qknorm_rope_kernel<64>, g, b, 0, s, qkv, ld, M, d, qgain, kgain, rope, dst_row, qo, ko, ldo, k_col_off, do_k, split, qgain2, kgain2, qscale);
  else hipLaunchKernelGGL(qknorm_rope_kernel<128>, g, b, 0, s, qkv, ld, M, d, qgain, kgain, rope, dst_row, qo, ko, ldo, k_col_off, do_k, split, qgain2, kgain2, qscale);
}

// ---------------------------------------------------------------------------------------
// V transpose: vt[h][c][col] = v[src_of_col[col]][v_col_off + h*dh + c]   (0 where src < 0)
// one workgroup per (64-column tile, head), through a padded LDS tile.
// ---------------------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256) void v_transpose_kernel(const bf16_t* __restrict__ v, int ld, int v_col_off,
                                                          const int* __restrict__ src_of_col,
                                                          bf16_t* __restrict__ vt, int ldvt) {
  __shared__ uint16_t tile[64][DH + 2];
  const int c0 = blockIdx.x * 64, h = blockIdx.y;
  const int tid = threadIdx.x;
  // load: 64 keys x DH values; a group of DH/2 threads reads one key row as 4-byte words
  constexpr int TPR = DH / 2;                 // threads per key row
  constexpr int RPP = 256 / TPR;              // key rows per pass
#pragma unroll
  for (int p = 0; p < 64 / RPP; ++p) {
    const int key = p * RPP + tid / TPR, w = tid % TPR;
    const int src = src_of_col[c0 + key];
    uint32_t raw = 0;
    if (src >= 0) raw = *(const uint32_t*)(v + (size_t)src * ld + v_col_off + h * DH + 2 * w);
    tile[key][2 * w] = (uint16_t)(raw & 0xFFFF);
    tile[key][2 * w + 1] = (uint16_t)(raw >> 16);
  }
  __syncthreads();
  // store: DH rows of 64 keys; 32 threads write one row as 4-byte words
#pragma unroll
  for (int p = 0; p < DH / 8; ++p) {
    const int c = p * 8 + tid / 32, w = tid % 32;
    const uint32_t out = (uint32_t)tile[2 * w][c] | ((uint32_t)tile[2 * w + 1][c] << 16);
    *(uint32_t*)(vt + ((size_t)h * DH + c) * ldvt + c0 + 2 * w) = out;
  }
}

void launch_v_transpose(hipStream_t s, const bf16_t* v, int ld, int v_col_off, int H, int dh,
                        const int* src_of_col, int n_cols_pad, bf16_t* vt, int ldvt) {
  if (n_cols_pad == 0) return;
  dim3 g(n_cols_pad / 64, H), b(256);
  if (dh == 64) hipLaunchKernelGGL(v_transpose_kernel<64>, g, b, 0, s, v, ld, v_col_off, src_of_col, vt, ldvt);
  else hipLaunchKernelGGL(v_transpose_kernel<128>, g, b, 0, s, v, ld, v_col_off, src_of_col, vt, ldvt);
}

// ---------------------------------------------------------------------------------------
// latent update  x <- a x + b v   (one span, scalar coefficients)
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void latent_update_kernel(float* __restrict__ x, const float* __restrict__ v,
                                                            long long n, float a, float b) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i < n) x[i] = a * x[i] + b * v[i];
}

void launch_latent_update(hipStream_t s, float* x, const float* v, long long n, float a, float b) {
  if (n == 0) return;
  hipLaunchKernelGGL(latent_update_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, x, v, n, a, b);
}

// ---------------------------------------------------------------------------------------
// small-M products  y[m][off_j + n] = sum_k f(x[m][k]) W_j[n][k] + bias_j[n]   (fp32 x, bf16 W, fp32 y)
// for a table of matrices W_j that share x: the conditioning vectors of a few (step, request) rows against
// the timestep MLP and the modulation matrices of every block (1.4 GB of weights at hidden 1536, read once).
// Grid (column groups, matrix).  A workgroup stages f(x) for up to MR rows in LDS once (SiLU included) and
// owns 32 columns, 8 per wave; a lane reads 16 bytes of a weight row per pass over K and the matching two
// 16-byte pieces of every staged row (even and odd pieces are kept in separate halves of the staged row, so
// that the lanes of a wave read consecutive LDS addresses).
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ float silu_f(float x) { return x / (1.f + __expf(-x)); }

template <int MR>
__global__ __launch_bounds__(256) void skinny_kernel(const float* __restrict__ x, int ldx, const SkinnyMat* __restrict__ mats,
                                                     float* __restrict__ y, int ldy, int M, int K, int silu_in) {
  extern __shared__ __attribute__((aligned(16))) float xs[];          // [MR][K]
  const SkinnyMat mt = mats[blockIdx.y];
  if ((int)blockIdx.x * 32 >= mt.N) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int n0 = blockIdx.x * 32 + wave * 8;
  const int KH = K >> 1;                                               // floats in the half that holds the even pieces
  for (int m0 = 0; m0 < M; m0 += MR) {
    const int rows = M - m0 < MR ? M - m0 : MR;
    __syncthreads();
    for (int idx = threadIdx.x * 4; idx < rows * K; idx += 1024) {
      const int r = idx / K, k = idx - r * K, q = k >> 2;
      float4 v = *(const float4*)(x + (size_t)(m0 + r) * ldx + k);
      if (silu_in) { v.x = silu_f(v.x); v.y = silu_f(v.y); v.z = silu_f(v.z); v.w = silu_f(v.w); }
      *(float4*)(xs + r * K + (q & 1) * KH + (q >> 1) * 4) = v;
    }
    __syncthreads();
    // four columns at a time: each staged piece is read once for four weight rows, and a lane has four
    // 16-byte weight loads in flight (these products run at memory latency)
    for (int c = 0; c < 8; c += 4) {
      if (n0 + c >= mt.N) break;
      const bf16_t* wr[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) wr[j] = mt.W + (size_t)(n0 + c + j < mt.N ? n0 + c + j : mt.N - 1) * mt.ldw;
      float acc[MR][4];
#pragma unroll
      for (int i = 0; i < MR; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
      for (int k = lane * 8; k < K; k += 512) {
        uint4 wraw[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) wraw[j] = *(const uint4*)(wr[j] + k);
        float w[4][8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          w[j][0] = bf2f((uint16_t)(wraw[j].x & 0xFFFF)); w[j][1] = bf2f((uint16_t)(wraw[j].x >> 16));
          w[j][2] = bf2f((uint16_t)(wraw[j].y & 0xFFFF)); w[j][3] = bf2f((uint16_t)(wraw[j].y >> 16));
          w[j][4] = bf2f((uint16_t)(wraw[j].z & 0xFFFF)); w[j][5] = bf2f((uint16_t)(wraw[j].z >> 16));
          w[j][6] = bf2f((uint16_t)(wraw[j].w & 0xFFFF)); w[j][7] = bf2f((uint16_t)(wraw[j].w >> 16));
        }
#pragma unroll
        for (int i = 0; i < MR; ++i) {
          if (i < rows) {
            const float4 xa = *(const float4*)(xs + i * K + (k >> 1)), xb = *(const float4*)(xs + i * K + KH + (k >> 1));
#pragma unroll
            for (int j = 0; j < 4; ++j)
              acc[i][j] += ((xa.x * w[j][0] + xa.y * w[j][1]) + (xa.z * w[j][2] + xa.w * w[j][3])) +
                           ((xb.x * w[j][4] + xb.y * w[j][5]) + (xb.z * w[j][6] + xb.w * w[j][7]));
          }
        }
      }
#pragma unroll
      for (int i = 0; i < MR; ++i) {
        if (i < rows) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float t = wave_sum(acc[i][j]);
            const int n = n0 + c + j;
            if (lane == 0 && n < mt.N) y[(size_t)(m0 + i) * ldy + mt.out_off + n] = t + (mt.bias ? mt.bias[n] : 0.f);
          }
        }
      }
    }
  }
}

// K a multiple of 8, ldx a multiple of 4, every ldw a multiple of 8; returns false when the shape is not one it takes
bool launch_skinny(hipStream_t s, const float* x, int ldx, const SkinnyMat* dev_mats, int n_mats, int max_n, float* y,
                   int ldy, int M, int K, int silu_in) {
  if (M == 0 || n_mats == 0 || max_n == 0) return true;
  if (K % 8 || ldx % 4 || K > 16384) return false;
  const dim3 g((max_n + 31) / 32, n_mats), b(256);
  // rows staged at a time: as many as 64 KB of LDS hold (fewer rows, less LDS, more workgroups per CU)
  auto lds = [&](int mr) { return (size_t)(M < mr ? M : mr) * K * 4; };
  if (K <= 2048) hipLaunchKernelGGL(skinny_kernel<8>, g, b, lds(8), s, x, ldx, dev_mats, y, ldy, M, K, silu_in);
  else if (K <= 4096) hipLaunchKernelGGL(skinny_kernel<4>, g, b, lds(4), s, x, ldx, dev_mats, y, ldy, M, K, silu_in);
  else if (K <= 8192) hipLaunchKernelGGL(skinny_kernel<2>, g, b, lds(2), s, x, ldx, dev_mats, y, ldy, M, K, silu_in);
  else hipLaunchKernelGGL(skinny_kernel<1>, g, b, lds(1), s, x, ldx, dev_mats, y, ldy, M, K, silu_in);
  return true;
}

// hi + lo = SiLU(x) (or x itself) as two bf16 terms (about 16 mantissa bits), for feeding an MFMA GEMM
__global__ __launch_bounds__(256) void silu_split_kernel(const float* __restrict__ x, bf16_t* __restrict__ hi,
                                                         bf16_t* __restrict__ lo, long long n, int silu) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const float v = silu ? silu_f(x[i]) : x[i];
  const uint16_t h = f2bf(v);
  hi[i] = h;
  lo[i] = f2bf(v - bf2f(h));
}
void launch_silu_split(hipStream_t s, const float* x, bf16_t* hi, bf16_t* lo, long long n, int silu) {
  if (n == 0) return;
  hipLaunchKernelGGL(silu_split_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, x, hi, lo, n, silu);
}

// ---------------------------------------------------------------------------------------
// Keys and values of a cross-attention from their fp32 product kv[rows][2d] (key columns, then
// value columns).  Keys: per-head RMS norm (eps 1e-6) times gain, stored as fp16 (a normalised
// key is bounded by sqrt(dh) max|gain|, far inside the fp16 range, and fp16 keeps three more
// mantissa bits than bf16).  Values: transposed, as two bf16 terms hi + lo:
// vt_*[h][c][col] = v[src_of_col[col]][h*dh + c]  (0 where src < 0).
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void cross_k_norm_kernel(const float* __restrict__ kv, int ld, int M, int H, int dh,
                                                           const float* __restrict__ gain, uint16_t* __restrict__ ko,
                                                           int ldo) {
  const int wave = (int)(((long long)blockIdx.x * 256 + threadIdx.x) >> 6), lane = threadIdx.x & 63;
  if (wave >= M * H) return;
  const int row = wave / H, h = wave - row * H;
  const float* src = kv + (size_t)row * ld + h * dh;
  const int per = dh >> 6;                      // 1 or 2 elements per lane
  float x[2] = {0.f, 0.f}, ss = 0.f;
  for (int e = 0; e < per; ++e) { x[e] = src[lane * per + e]; ss += x[e] * x[e]; }
  ss = wave_sum(ss);
  const float r = rsqrtf(ss / (float)dh + 1e-6f);
  for (int e = 0; e < per; ++e) {
    const _Float16 hv = (_Float16)(x[e] * r * gain[lane * per + e]);
    ko[(size_t)row * ldo + h * dh + lane * per + e] = *(const uint16_t*)&hv;
  }
}
__global__ __launch_bounds__(256) void cross_vt_split_kernel(const float* __restrict__ kv, int ld, int v_col_off, int dh,
                                                             const int* __restrict__ src_of_col,
                                                             bf16_t* __restrict__ vt_hi, bf16_t* __restrict__ vt_lo,
                                                             int ldvt) {
  const int c0 = blockIdx.x * 64, h = blockIdx.y;
  const int col = threadIdx.x & 63, cg = threadIdx.x >> 6;
  const int src = src_of_col[c0 + col];
  for (int c = cg; c < dh; c += 4) {
    const float v = src >= 0 ? kv[(size_t)src * ld + v_col_off + h * dh + c] : 0.f;
    const uint16_t hi = f2bf(v);
    const size_t o = ((size_t)h * dh + c) * ldvt + c0 + col;
    vt_hi[o] = hi;
    vt_lo[o] = f2bf(v - bf2f(hi));
  }
}
void launch_cross_kv_finish(hipStream_t s, const float* kv, int ld, int M, int H, int dh, const float* kgain,
                            bf16_t* k16, int ldk, const int* src_of_col, int n_cols_pad, bf16_t* vt_hi,
                            bf16_t* vt_lo, int ldvt) {
  if (M == 0) return;
  const long long waves = (long long)M * H;
  hipLaunchKernelGGL(cross_k_norm_kernel, dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, s, kv, ld, M, H, dh, kgain,
                     (uint16_t*)k16, ldk);
  if (n_cols_pad > 0)
    hipLaunchKernelGGL(cross_vt_split_kernel, dim3(n_cols_pad / 64, H), dim3(256), 0, s, kv, ld, H * dh, dh, src_of_col,
                       vt_hi, vt_lo, ldvt);
}

// out[m][0..127] = cos(1000 sigma f_k), out[m][128..255] = sin(...), f_k = exp(-ln(1e4) k/128)
__global__ void timestep_features_kernel(const float* __restrict__ sigma, float* __restrict__ out, int M) {
  const int m = blockIdx.x, k = threadIdx.x;   // 128 threads
  if (m >= M) return;
  const float f = expf(-9.210340371976184f * (float)k / 128.f);
  const float ang = 1000.f * sigma[m] * f;
  out[(size_t)m * 256 + k] = cosf(ang);
  out[(size_t)m * 256 + 128 + k] = sinf(ang);
}
void launch_timestep_features(hipStream_t s, const float* sigma_dev, float* out, int M) {
  if (M == 0) return;
  hipLaunchKernelGGL(timestep_features_kernel, dim3(M), dim3(128), 0, s, sigma_dev, out, M);
}

// ---------------------------------------------------------------------------------------
// patchify: token t of request r, feature ((c*pt+dt)*ph+dh)*pw+dw  <-  latent[c][f][y][x]
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void patchify_kernel(const float* __restrict__ lat,
                                                       const long long* __restrict__ lat_off,
                                                       const int4* __restrict__ req_dims,
                                                       const TokInfo* __restrict__ tok, int n_img, int C,
                                                       int pt, int ph, int pw, bf16_t* __restrict__ out,
                                                       bf16_t* __restrict__ out_lo, int ldp) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long long)n_img * ldp) return;
  const int t = (int)(idx / ldp), feat = (int)(idx % ldp);
  const int pdim = C * pt * ph * pw;
  float v = 0.f;
  if (feat < pdim) {
    const TokInfo ti = tok[t];
    const int4 dm = req_dims[ti.req];          // (F, H, W, -)
    int dw = feat % pw, r = feat / pw;
    int dh = r % ph; r /= ph;
    int dt = r % pt; const int c = r / pt;
    const int f = ti.f * pt + dt, yy = ti.i * ph + dh, xx = ti.j * pw + dw;
    v = lat[lat_off[ti.req] + (((long long)c * dm.x + f) * dm.y + yy) * dm.z + xx];
  }
  const uint16_t hi = f2bf(v);
  out[idx] = hi;
  out_lo[idx] = f2bf(v - bf2f(hi));     // latent = hi + lo to about 16 mantissa bits
}
void launch_patchify(hipStream_t s, const float* lat, const long long* lat_off_dev, const int4* req_dims_dev,
                     const TokInfo* tok, int n_img, int C, int pt, int ph, int pw, bf16_t* out, bf16_t* out_lo,
                     int ldp) {
  const long long total = (long long)n_img * ldp;
  if (total == 0) return;
  hipLaunchKernelGGL(patchify_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, lat, lat_off_dev,
                     req_dims_dev, tok, n_img, C, pt, ph, pw, out, out_lo, ldp);
}

// x[t][c] += PE(i, j)[c]:  quarters [sin(i w), cos(i w), sin(j w), cos(j w)], w_k = 1e4^(-k/(d/4))
__global__ __launch_bounds__(256) void add_pe_kernel(float* __restrict__ x, const TokInfo* __restrict__ tok,
                                                     int n_img, int d) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long long)n_img * d) return;
  const int t = (int)(idx / d), c = (int)(idx % d);
  const int qd = d >> 2, part = c / qd, k = c % qd;
  const TokInfo ti = tok[t];
  const float w = exp2f(-13.287712379549449f * (float)k / (float)qd);   // log2(1e4)
  const float ang = (float)(part < 2 ? ti.i : ti.j) * w;
  x[idx] += (part & 1) ? cosf(ang) : sinf(ang);
}
void launch_add_pe(hipStream_t s, float* x, const TokInfo* tok, int n_img, int d) {
  const long long total = (long long)n_img * d;
  if (total == 0) return;
  hipLaunchKernelGGL(add_pe_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, x, tok, n_img, d);
}

// ---------------------------------------------------------------------------------------
// unpatchify + latent update: every latent element looks up its token/feature in y
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void unpatchify_update_kernel(float* __restrict__ lat, float* __restrict__ v_out,
                                                                const float* __restrict__ y, int ldy,
                                                                const long long* __restrict__ lat_off,
                                                                const int4* __restrict__ req_dims,
                                                                const int* __restrict__ img_off,
                                                                const float* __restrict__ a, const float* __restrict__ b,
                                                                int n_req, long long total, int C, int pt, int ph, int pw) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  int r = 0;
  while (r + 1 < n_req && idx >= lat_off[r + 1]) ++r;
  const int4 dm = req_dims[r];
  long long e = idx - lat_off[r];
  const int xx = (int)(e % dm.z); e /= dm.z;
  const int yy = (int)(e % dm.y); e /= dm.y;
  const int f = (int)(e % dm.x); const int c = (int)(e / dm.x);
  const int gh = dm.y / ph, gw = dm.z / pw;
  const int tokl = ((f / pt) * gh + yy / ph) * gw + xx / pw;
  const int feat = ((c * pt + f % pt) * ph + yy % ph) * pw + xx % pw;
  const float v = y[(size_t)(img_off[r] + tokl) * ldy + feat];
  if (v_out) v_out[idx] = v;
  lat[idx] = a[r] * lat[idx] + b[r] * v;
}
void launch_unpatchify_update(hipStream_t s, float* lat, float* v_out, const float* y, int ldy,
                              const long long* lat_off_dev, const int4* req_dims_dev, const int* img_off_dev,
                              const float* a_dev, const float* b_dev, int n_req, long long total, int C, int pt,
                              int ph, int pw) {
  if (total == 0) return;
  hipLaunchKernelGGL(unpatchify_update_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, lat, v_out, y,
                     ldy, lat_off_dev, req_dims_dev, img_off_dev, a_dev, b_dev, n_req, total, C, pt, ph, pw);
}

// ---------------------------------------------------------------------------------------
// rotary table: out[row][j] = (cos, sin)(pos_axis * theta^(-2 jj / D_axis)); rows that are
// not image tokens (tok_of_row < 0) get the identity rotation.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void rope_table_kernel(const TokInfo* __restrict__ tok,
                                                         const int* __restrict__ tok_of_row, int n_rows, int dh,
                                                         int ax0, int ax1, int ax2, float log2_theta,
                                                         float2* __restrict__ out) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  const int hp = dh >> 1;
  if (idx >= (long long)n_rows * hp) return;
  const int row = (int)(idx / hp), j = (int)(idx % hp);
  const int t = tok_of_row ? tok_of_row[row] : row;
  float2 cs = make_float2(1.f, 0.f);
  if (t >= 0) {
    const TokInfo ti = tok[t];
    int e = 2 * j, width, pos;
    if (e < ax0) { width = ax0; pos = ti.f; }
    else if (e < ax0 + ax1) { e -= ax0; width = ax1; pos = ti.i; }
    else { e -= ax0 + ax1; width = ax2; pos = ti.j; }
    const float freq = exp2f(-log2_theta * (float)e / (float)width);
    const float ang = (float)pos * freq;
    cs = make_float2(cosf(ang), sinf(ang));
  }
  out[idx] = cs;
}
void launch_rope_table(hipStream_t s, const TokInfo* tok, const int* tok_of_row, int n_rows, int dh, int ax0,
                       int ax1, int ax2, float theta, float2* out) {
  const long long total = (long long)n_rows * (dh / 2);
  if (total == 0) return;
  hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, tok, tok_of_row,
                     n_rows, dh, ax0, ax1, ax2, log2f(theta), out);
}

// out[m][n] = base[m][n] + table[n]
__global__ __launch_bounds__(256) void add_rows_kernel(const float* __restrict__ base, int ld_base,
                                                       const float* __restrict__ table, float* __restrict__ out,
                                                       int ld_out, int M, int N) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long long)M * N) return;
  const int m = (int)(idx / N), n = (int)(idx % N);
  out[(size_t)m * ld_out + n] = base[(size_t)m * ld_base + n] + table[n];
}
void launch_add_rows(hipStream_t s, const float* base, int ld_base, const float* table, float* out, int ld_out,
                     int M, int N) {
  const long long total = (long long)M * N;
  if (total == 0) return;
  hipLaunchKernelGGL(add_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, base, ld_base, table,
                     out, ld_out, M, N);
}

// dst[dst_row[m]][:] = src[src_row[m]][:]   (float4 granules, d % 4 == 0)
__global__ __launch_bounds__(256) void copy_rows_kernel(const float4* __restrict__ src, const int* __restrict__ src_row,
                                                        float4* __restrict__ dst, const int* __restrict__ dst_row,
                                                        int M, int d4) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long long)M * d4) return;
  const int m = (int)(idx / d4), c = (int)(idx % d4);
  const int sr = src_row ? src_row[m] : m, dr = dst_row ? dst_row[m] : m;
  dst[(size_t)dr * d4 + c] = src[(size_t)sr * d4 + c];
}
void launch_copy_rows_f32(hipStream_t s, const float* src, const int* src_row, float* dst, const int* dst_row,
                          int M, int d) {
  const long long total = (long long)M * (d / 4);
  if (total == 0) return;
  hipLaunchKernelGGL(copy_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const float4*)src,
                     src_row, (float4*)dst, dst_row, M, d / 4);
}

// ---------------------------------------------------------------------------------------
// weight initialisation: counter-based Gaussian, float64 Box-Muller (so that an independent
// float64 host implementation of the same recipe produces bit-identical bf16 values)
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t mix64(uint64_t x) {
  uint64_t z = x + 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
__device__ __forceinline__ float gauss(uint64_t key, uint64_t i, double std) {
  const uint64_t z = mix64(key + i);
  const double u1 = ((double)(z >> 40) + 1.0) * (1.0 / 16777216.0);
  const double u2 = (double)((z >> 16) & 0xFFFFFFull) * (1.0 / 16777216.0);
  const double g = sqrt(-2.0 * log(u1)) * cos(6.283185307179586 * u2);
  return (float)(std * g);
}
// stored [rows_out][ldw]; logical element (in i, out o) has index i*rows_out + o
__global__ __launch_bounds__(256) void init_matrix_kernel(bf16_t* __restrict__ w, int rows_out, int cols_in, int ldw,
                                                          uint64_t key, float std) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long long)rows_out * cols_in) return;
  const int o = (int)(idx / cols_in), i = (int)(idx % cols_in);
  w[(size_t)o * ldw + i] = f2bf(gauss(key, (uint64_t)i * rows_out + o, (double)std));
}
void launch_init_matrix(hipStream_t s, bf16_t* w, int rows_out, int cols_in, int ldw, uint64_t key, float std) {
  const long long total = (long long)rows_out * cols_in;
  if (total == 0) return;
  hipLaunchKernelGGL(init_matrix_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, w, rows_out,
                     cols_in, ldw, key, std);
}
__global__ __launch_bounds__(256) void init_table_kernel(float* __restrict__ w, long long n, uint64_t key, float std) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= n) return;
  w[idx] = bf2f(f2bf(gauss(key, (uint64_t)idx, (double)std)));
}
void launch_init_table_f32(hipStream_t s, float* w, long long n, uint64_t key, float std) {
  if (n == 0) return;
  hipLaunchKernelGGL(init_table_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, w, n, key, std);
}
__global__ __launch_bounds__(256) void fill_f32_kernel(float* p, long long n, float v) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx < n) p[idx] = v;
}
void launch_fill_f32(hipStream_t s, float* p, long long n, float v) {
  if (n == 0) return;
  hipLaunchKernelGGL(fill_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, n, v);
}
__global__ __launch_bounds__(256) void fill_u16_kernel(uint16_t* p, long long n, uint16_t v) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx < n) p[idx] = v;
}
void launch_fill_u16(hipStream_t s, bf16_t* p, long long n, uint16_t v) {
  if (n == 0) return;
  hipLaunchKernelGGL(fill_u16_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, n, v);
}

}  // namespace dit
