// Row-wise kernels of the Encode stage (T5-v1.1-style text encoder): embedding lookup, RMS
// norm, the gated-GELU product and the relative-position bias table.  The matrix products and
// the attention of the stage run in gemm.hip / attention.hip.
#include "dit_internal.h"

namespace dit {

namespace {
__device__ __forceinline__ uint16_t e_f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float e_bf2f(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ uint32_t e_pack2(float a, float b) { return (uint32_t)e_f2bf(a) | ((uint32_t)e_f2bf(b) << 16); }
__device__ __forceinline__ float e_wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
}  // namespace

// x[m][:] = table[token[m]][:]   (fp32 table rows, d a multiple of 4; out-of-range ids read row 0)
__global__ __launch_bounds__(256) void embed_gather_kernel(const int* __restrict__ tokens, const float* __restrict__ table,
                                                           float* __restrict__ x, int M, int d, int vocab) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;      // one float4 each
  const int per = d >> 2;
  if (i >= (long long)M * per) return;
  const int m = (int)(i / per), c = (int)(i % per);
  int t = tokens[m];
  if (t < 0 || t >= vocab) t = 0;
  ((float4*)x)[i] = ((const float4*)(table + (size_t)t * d))[c];
}

void launch_embed_gather(hipStream_t s, const int* tokens, const float* table, float* x, int M, int d, int vocab) {
  if (M == 0) return;
  const long long n = (long long)M * (d / 4);
  hipLaunchKernelGGL(embed_gather_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, tokens, table, x, M, d, vocab);
}

// y = x / sqrt(mean(x^2) + 1e-6) * gain  (no mean subtraction): bf16 y and/or fp32 y32.
// One wave per row, the row stays in registers between the reduction and the scaling.
template <int MAXV>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float* __restrict__ x, const float* __restrict__ gain,
                                                      bf16_t* __restrict__ y, float* __restrict__ y32, int M, int d) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= M) return;
  const int lane = threadIdx.x & 63;
  const int nv = d >> 8;
  const float4* xr = (const float4*)(x + (size_t)row * d);
  float4 v[MAXV];
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < MAXV; ++i)
    if (i < nv) {
      v[i] = xr[i * 64 + lane];
      q += (v[i].x * v[i].x + v[i].y * v[i].y) + (v[i].z * v[i].z + v[i].w * v[i].w);
    }
  const float r = rsqrtf(e_wave_sum(q) / (float)d + 1e-6f);
#pragma unroll
  for (int i = 0; i < MAXV; ++i)
    if (i < nv) {
      const float4 g = ((const float4*)gain)[i * 64 + lane];
      const float r0 = v[i].x * r * g.x, r1 = v[i].y * r * g.y, r2 = v[i].z * r * g.z, r3 = v[i].w * r * g.w;
      if (y) {
        uint2 w;
        w.x = e_pack2(r0, r1); w.y = e_pack2(r2, r3);
        ((uint2*)(y + (size_t)row * d))[i * 64 + lane] = w;
      }
      if (y32) ((float4*)(y32 + (size_t)row * d))[i * 64 + lane] = make_float4(r0, r1, r2, r3);
    }
}

void launch_rmsnorm(hipStream_t s, const float* x, const float* gain, bf16_t* y, float* y32, int M, int d) {
  if (M == 0) return;
  dim3 g((M + 3) / 4), b(256);
  if (d <= 1024) hipLaunchKernelGGL(rmsnorm_kernel<4>, g, b, 0, s, x, gain, y, y32, M, d);
  else if (d <= 4096) hipLaunchKernelGGL(rmsnorm_kernel<16>, g, b, 0, s, x, gain, y, y32, M, d);
  else hipLaunchKernelGGL(rmsnorm_kernel<32>, g, b, 0, s, x, gain, y, y32, M, d);
}

// act = gelu_tanh(a) * b   elementwise on bf16, 8 elements per thread
__global__ __launch_bounds__(256) void geglu_kernel(const bf16_t* __restrict__ a, const bf16_t* __restrict__ b,
                                                    bf16_t* __restrict__ out, long long n8) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= n8) return;
  const uint4 ra = ((const uint4*)a)[i], rb = ((const uint4*)b)[i];
  const uint32_t wa[4] = {ra.x, ra.y, ra.z, ra.w}, wb[4] = {rb.x, rb.y, rb.z, rb.w};
  uint32_t wo[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    float r[2];
#pragma unroll
    for (int hlf = 0; hlf < 2; ++hlf) {
      const float x = e_bf2f((uint16_t)(hlf ? wa[p] >> 16 : wa[p] & 0xFFFF));
      const float y = e_bf2f((uint16_t)(hlf ? wb[p] >> 16 : wb[p] & 0xFFFF));
      // 0.5 x (1 + tanh(u)) = x / (1 + exp(-2u)), u = sqrt(2/pi) (x + 0.044715 x^3)
      const float t = x * (0.7978845608028654f + 0.035677408136300125f * x * x);
      r[hlf] = x * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-2.8853900817779268f * t)) * y;
    }
    wo[p] = e_pack2(r[0], r[1]);
  }
  ((uint4*)out)[i] = make_uint4(wo[0], wo[1], wo[2], wo[3]);
}

void launch_geglu(hipStream_t s, const bf16_t* a, const bf16_t* b, bf16_t* out, long long n) {
  if (n == 0) return;
  const long long n8 = n / 8;                                   // n is a multiple of 8 (row length is)
  hipLaunchKernelGGL(geglu_kernel, dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, s, a, b, out, n8);
}

// bias[h][delta + L - 1] = table[bucket(delta)][h], delta = key position - query position in
// (-L, L): the encoder's 32 relative-position buckets, 16 per direction, of which 8 are exact
// (distance 0..7) and 8 logarithmic up to distance 128: 8 + floor(8 ln(n/8) / ln 16), taken
// here as the number of b in 1..7 with n^2 >= 64 * 2^b (the same inequality squared, exact in
// integers); distances from 128 on share bucket 15.
__global__ __launch_bounds__(256) void rel_bias_table_kernel(const float* __restrict__ table, float* __restrict__ bias,
                                                             int H, int L) {
  const int span = 2 * L - 1;
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= H * span) return;
  const int h = i / span, delta = i % span - (L - 1);
  const int n = delta < 0 ? -delta : delta;
  int bucket;
  if (n < 8) bucket = n;
  else if (n >= 128) bucket = 15;
  else {
    bucket = 8;
    for (int b = 1; b < 8; ++b) bucket += (n * n >= (64 << b)) ? 1 : 0;
  }
  if (delta > 0) bucket += 16;
  bias[i] = table[bucket * H + h];
}

void launch_rel_bias_table(hipStream_t s, const float* table, float* bias, int H, int L) {
  const int n = H * (2 * L - 1);
  if (n <= 0) return;
  hipLaunchKernelGGL(rel_bias_table_kernel, dim3((n + 255) / 256), dim3(256), 0, s, table, bias, H, L);
}

}  // namespace dit
