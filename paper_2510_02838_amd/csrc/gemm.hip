// bf16 GEMM on the gfx950 matrix cores:  C[M][N] = A[M][K] * W[N][K]^T  (+ epilogue).
//
// Used for every dense contraction of the denoising step except attention: QKV, attention
// output projection, both MLP matmuls, the embeddings and the final projection.
//
// Tiling.  A workgroup owns a BM x BN tile of C and walks K in slabs of 64.  Slabs of A and
// W go from global memory straight into LDS (global_load_lds_dwordx4: each lane deposits 16
// bytes at wave-base + 16*lane, no staging registers), double buffered with one barrier per
// slab.  Which 16-byte chunk a lane fetches is XOR-swizzled on the global side, so that the
// 128-bit LDS reads that feed the MFMA operands are bank-conflict free.  (DIRECT = false
// keeps a register-staged copy path, for comparison.)  A wave owns a (BM/WM) x (BN/WN) sub-tile made of 32x32 MFMA tiles
// (v_mfma_f32_32x32x16_bf16: 64 lanes, A operand = 32 rows x 16 k, B operand = 16 k x 32
// columns, each lane supplies 8 consecutive k).  MFMA rows are rows of A (tokens), MFMA
// columns are rows of W (output features), so the 32 lanes of a half-wave write 32
// consecutive output features of one token.
//
// Several problems (for example the text and the image stream of one joint block, which
// have different weights) are launched as one grid.  Workgroup ids are first de-interleaved
// over the 8 XCDs (ids are dealt round-robin to XCDs by the hardware) so that workgroups
// sharing an L2 work on neighbouring tiles, then mapped to tiles in groups of 8 tile rows.
#include "dit_internal.h"
#include <type_traits>

namespace dit {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

static constexpr int BK = 64;          // k-slab, elements
static constexpr int ROW_BYTES = 128;  // one slab row in LDS

__device__ __forceinline__ uint16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float gelu_tanh(float x) {
  // 0.5 x (1 + tanh(u)) == x * sigmoid(2u),  u = sqrt(2/pi) (x + 0.044715 x^3)
  float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
  return x / (1.0f + __expf(-2.0f * u));
}

// byte offset of 16-byte chunk `c` (0..7) of slab row `r`
__device__ __forceinline__ int swz(int r, int c) { return r * ROW_BYTES + ((c ^ ((r >> 1) & 7)) << 4); }

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

template <int BM, int BN, int WM, int WN, bool DIRECT>
__global__ __launch_bounds__(WM * WN * 64) void gemm_kernel(const GemmBatch batch) {
  constexpr int NT = WM * WN * 64;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr int LA = BM * 8 / NT, LB = BN * 8 / NT;   // 16-byte chunks per thread per slab
  static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile/threads");
  extern __shared__ __attribute__((aligned(128))) unsigned char smem[];
  constexpr int STAGE = (BM + BN) * ROW_BYTES;   // one slab of A then one slab of W
  constexpr int OFFB = BM * ROW_BYTES;

  // ---- workgroup -> (problem, tile) ----------------------------------------------------
  int bid = blockIdx.x, nb = gridDim.x;
  {
    int x = bid & 7, idx = bid >> 3, q = nb >> 3, rem = nb & 7;
    bid = x * q + (x < rem ? x : rem) + idx;
  }
  GemmProblem P = batch.p[0];   // static indices only: keeps the argument block in SGPRs
  if (batch.n > 1 && bid >= batch.p[1].tile_start) P = batch.p[1];
  if (batch.n > 2 && bid >= batch.p[2].tile_start) P = batch.p[2];
  int t = bid - P.tile_start;
  int tm, tn;
  {
    constexpr int GM = 8;
    int per = GM * P.tiles_n;
    int g = t / per, r = t - g * per;
    int first = g * GM;
    int gsz = P.tiles_m - first < GM ? P.tiles_m - first : GM;
    tm = first + r % gsz;
    tn = r / gsz;
  }
  const int m0 = tm * BM, n0 = tn * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  // ---- per-thread global source pointers -----------------------------------------------
  // (element offsets from the matrix base; every operand is far below 2^31 elements)
  uint32_t ga[LA], gb[LB];
#pragma unroll
  for (int i = 0; i < LA; ++i) {
    int q = i * NT + tid, r = q >> 3, pc = q & 7, c = pc ^ ((r >> 1) & 7);
    int m = m0 + r; if (m >= P.M) m = P.M - 1;            // clamp: rows past M are never stored
    ga[i] = (uint32_t)m * (uint32_t)P.lda + c * 8;
  }
#pragma unroll
  for (int i = 0; i < LB; ++i) {
    int q = i * NT + tid, r = q >> 3, pc = q & 7, c = pc ^ ((r >> 1) & 7);
    gb[i] = (uint32_t)(n0 + r) * (uint32_t)P.ldw + c * 8; // weights are padded to N_pad rows
  }

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int nk = P.K / BK;
  const int arow = wm * (BM / WM) + (lane & 31);
  const int brow = wn * (BN / WN) + (lane & 31);
  const int half = lane >> 5;

  auto compute = [&](const unsigned char* cA, const unsigned char* cB) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      bf16x8 a[TM], b[TN];
      const int c = kk * 2 + half;
#pragma unroll
      for (int i = 0; i < TM; ++i) a[i] = *(const bf16x8*)(cA + swz(arow + i * 32, c));
#pragma unroll
      for (int j = 0; j < TN; ++j) b[j] = *(const bf16x8*)(cB + swz(brow + j * 32, c));
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  };

  if constexpr (DIRECT) {
    // chunk q = i*NT + tid lands at LDS byte q*16 = (i*NT + wave*64)*16 + lane*16
    auto issue = [&](int kt, unsigned char* dA) {
      const bf16_t* Ak = P.A + kt * BK;
      const bf16_t* Wk = P.W + kt * BK;
      unsigned char* dB = dA + OFFB;
#pragma unroll
      for (int i = 0; i < LA; ++i)
        __builtin_amdgcn_global_load_lds((gptr_t)(Ak + ga[i]), (lptr_t)(dA + (i * NT + wave * 64) * 16), 16, 0, 0);
#pragma unroll
      for (int i = 0; i < LB; ++i)
        __builtin_amdgcn_global_load_lds((gptr_t)(Wk + gb[i]), (lptr_t)(dB + (i * NT + wave * 64) * 16), 16, 0, 0);
    };
    issue(0, smem);
    for (int kt = 0; kt < nk; ++kt) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // my part of slab kt has landed
      __syncthreads();                                   // everyone's has; slab kt-1 is free
      if (kt + 1 < nk) issue(kt + 1, smem + ((kt + 1) & 1) * STAGE);
      const unsigned char* cA = smem + (kt & 1) * STAGE;
      compute(cA, cA + OFFB);
    }
  } else {
    u32x4 ra[LA], rb[LB];
#pragma unroll
    for (int i = 0; i < LA; ++i) ra[i] = *(const u32x4*)(P.A + ga[i]);
#pragma unroll
    for (int i = 0; i < LB; ++i) rb[i] = *(const u32x4*)(P.W + gb[i]);
#pragma unroll
    for (int i = 0; i < LA; ++i) *(u32x4*)(smem + (i * NT + tid) * 16) = ra[i];
#pragma unroll
    for (int i = 0; i < LB; ++i) *(u32x4*)(smem + OFFB + (i * NT + tid) * 16) = rb[i];
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
      const unsigned char* cA = smem + (kt & 1) * STAGE;
      unsigned char* nA = smem + ((kt & 1) ^ 1) * STAGE;
      {
        // prefetch the next slab (the last iteration re-reads its own slab; the copy is unused)
        const int ko = (kt + 1 < nk ? kt + 1 : kt) * BK;
        const bf16_t* Ak = P.A + ko;
        const bf16_t* Wk = P.W + ko;
#pragma unroll
        for (int i = 0; i < LA; ++i) ra[i] = *(const u32x4*)(Ak + ga[i]);
#pragma unroll
        for (int i = 0; i < LB; ++i) rb[i] = *(const u32x4*)(Wk + gb[i]);
      }
      compute(cA, cA + OFFB);
#pragma unroll
      for (int i = 0; i < LA; ++i) *(u32x4*)(nA + (i * NT + tid) * 16) = ra[i];
#pragma unroll
      for (int i = 0; i < LB; ++i) *(u32x4*)(nA + OFFB + (i * NT + tid) * 16) = rb[i];
      __syncthreads();
    }
  }

  // ---- epilogue ---------------------------------------------------------------------------
  // acc[i][j][e] is C[mb + 8*(e/4) + (e%4)][n]: lanes 0..31 hold 32 consecutive n.
  auto epilogue = [&](auto kind_tag) {
    constexpr int KIND = decltype(kind_tag)::value;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = n0 + wn * (BN / WN) + j * 32 + (lane & 31);
      if (n < P.N) {
        const float bv = P.bias ? P.bias[n] : 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          const int mb = m0 + wm * (BM / WM) + i * 32 + 4 * half;
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int m = mb + 8 * (e >> 2) + (e & 3);
            if (m < P.M) {
              float v = acc[i][j][e] + bv;
              const size_t o = (size_t)m * P.ldc + n;
              if (KIND == OUT_BF16) {
                ((bf16_t*)P.out)[o] = f2bf(v);
              } else if (KIND == OUT_F32) {
                ((float*)P.out)[o] = v;
              } else if (KIND == OUT_GELU_BF16) {
                ((bf16_t*)P.out)[o] = f2bf(gelu_tanh(v));
              } else {
                float g = 1.f;
                if (P.gate) g = P.gate[(size_t)(P.row_req ? P.row_req[m] : 0) * P.gate_stride + n];
                ((float*)P.out)[o] += g * v;
              }
            }
          }
        }
      }
    }
  };
  if (P.out_kind == OUT_BF16) epilogue(std::integral_constant<int, OUT_BF16>{});
  else if (P.out_kind == OUT_F32) epilogue(std::integral_constant<int, OUT_F32>{});
  else if (P.out_kind == OUT_GELU_BF16) epilogue(std::integral_constant<int, OUT_GELU_BF16>{});
  else epilogue(std::integral_constant<int, OUT_RESID_F32>{});
}

template <int BM, int BN, int WM, int WN, bool DIRECT>
static void launch_t(hipStream_t s, GemmBatch& b) {
  int total = 0;
  for (int i = 0; i < b.n; ++i) {
    GemmProblem& p = b.p[i];
    p.tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.N + BN - 1) / BN;
    p.tile_start = total;
    total += p.tiles_m * p.tiles_n;
  }
  b.total_tiles = total;
  if (total == 0) return;
  size_t lds = 2 * (BM + BN) * ROW_BYTES;
  auto kern = gemm_kernel<BM, BN, WM, WN, DIRECT>;
  static bool attr_done = false;
  if (!attr_done) {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, dim3(total), dim3(WM * WN * 64), lds, s, b);
}

// variant codes: BM*1000 + BN, +1e6 for 8 waves (2x4), +2e6 for the register-staged path
int launch_gemm(hipStream_t s, GemmBatch& b, int force_tile) {
  // Tile choice: the big tile has the best MFMA-per-byte ratio but needs enough tiles to
  // fill 256 CUs; otherwise fall back to smaller tiles.
  int tile = force_tile;
  if (!tile) {
    long long t256 = 0;
    for (int i = 0; i < b.n; ++i)
      t256 += (long long)((b.p[i].M + 255) / 256) * ((b.p[i].N + 255) / 256);
    tile = (t256 >= 480) ? 256256 : 128128;
  }
  switch (tile) {
    case 256256: launch_t<256, 256, 2, 2, true>(s, b); break;
    case 1256256: launch_t<256, 256, 2, 4, true>(s, b); break;
    case 2256256: launch_t<256, 256, 2, 2, false>(s, b); break;
    case 256128: launch_t<256, 128, 2, 2, true>(s, b); break;
    case 128256: launch_t<128, 256, 2, 2, true>(s, b); break;
    case 2128128: launch_t<128, 128, 2, 2, false>(s, b); break;
    default: tile = 128128; launch_t<128, 128, 2, 2, true>(s, b); break;
  }
  return tile;
}

}  // namespace dit
