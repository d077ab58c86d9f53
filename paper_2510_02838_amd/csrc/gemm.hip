// bf16 GEMM on the gfx950 matrix cores:  C[M][N] = A[M][K] * W[N][K]^T  (+ epilogue).
//
// Used for every dense contraction of the denoising step except attention: QKV, attention
// output projection, both MLP matmuls, the embeddings and the final projection.
//
// Tiling.  A workgroup owns a BM x BN tile of C and walks K in slabs of BK (32 or 64).  Slabs
// of A and W go from global memory straight into LDS (global_load_lds_dwordx4: each lane
// deposits 16 bytes at wave-base + 16*lane, no staging registers) into a ring of NS stages.
// Which 16-byte chunk a lane fetches is XOR-swizzled on the global side, so that the 128-bit
// LDS reads that feed the MFMA operands are bank-conflict free (LDS on gfx950 serves 16 lanes
// x 16 bytes per clock from 64 banks: 16 consecutive slab rows must fall into 16 distinct
// 16-byte slots of a 256-byte window; the key is (row >> 1) & 7 for 128-byte rows and
// (row >> 2) & 3 for 64-byte rows).  A wave owns a (BM/WM) x (BN/WN) sub-tile made of 32x32
// MFMA tiles (v_mfma_f32_32x32x16_bf16: 64 lanes, A operand = 32 rows x 16 k, B operand =
// 16 k x 32 columns, each lane supplies 8 consecutive k).  MFMA rows are rows of A (tokens),
// MFMA columns are rows of W (output features), so the 32 lanes of a half-wave write 32
// consecutive output features of one token.
//
// Pipeline.  NS-1 slabs are in flight from global memory while one is computed: measured on
// MI355X a 64 KB slab takes about 1.4 us from issue to landing, as long as its MFMA work, so
// a single slab in flight leaves the matrix cores waiting.  Operand fragments are double
// buffered in registers: while the MFMAs of k-step kk run, the fragments of kk+1 are read
// from LDS.  The one barrier per slab sits before the slab's last k-step: by then every wave
// holds the slab's last fragments in registers, so the slab's stage is free for the loads of
// slab+NS, and the next slab becomes visible, so the last k-step already prefetches the next
// slab's first fragments.
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


__device__ __forceinline__ uint16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
// two floats -> packed bf16 pair, round-to-nearest-even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack2bf(float a, float b) {
  f32x2 v = {a, b};
  bf16x2 r = __builtin_convertvector(v, bf16x2);
  return *(uint32_t*)&r;
}

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
// two floats -> packed fp16 pair, round-to-nearest-even
__device__ __forceinline__ uint32_t pack2h(float a, float b) {
  f32x2 v = {a, b};
  f16x2 r = __builtin_convertvector(v, f16x2);
  return *(uint32_t*)&r;
}

__device__ __forceinline__ float gelu_tanh(float x) {
  // 0.5 x (1 + tanh(u)) == x * sigmoid(2u) == x / (1 + 2^(-2 log2(e) u)),
  // u = sqrt(2/pi) (x + 0.044715 x^3); hardware exp2 and reciprocal (1 ulp each)
  const float t = x * (0.7978845608028654f + 0.035677408136300125f * x * x);
  const float e = __builtin_amdgcn_exp2f(-2.8853900817779268f * t);
  return x * __builtin_amdgcn_rcpf(1.0f + e);
}

template <int BKT>
__device__ __forceinline__ int swz_key(int r) { return BKT == 64 ? ((r >> 1) & 7) : ((r >> 2) & 3); }

typedef __attribute__((address_space(3))) void* lptr_t;

#define SGB(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)
// scheduling hint for one k-step: NR LDS reads spread over NM MFMAs
template <int NR, int NM>
__device__ __forceinline__ void interleave_hint() {
  if constexpr (NM >= 16) {
    // one wave per SIMD: nothing else covers LDS latency, so all reads go out in the first half
#pragma unroll
    for (int i = 0; i < NR; ++i) {
      SGB(0x100, 1);
      SGB(0x008, 1);
    }
    SGB(0x008, NM - NR);
    return;
  }
  constexpr int per = NM / NR, extra = NM - per * NR;
#pragma unroll
  for (int i = 0; i < NR; ++i) {
    SGB(0x100, 1);      // one DS read
    SGB(0x008, per);    // `per` MFMAs
  }
  if (extra > 0) SGB(0x008, extra);
}
// s_waitcnt immediate for "at most N vector-memory loads outstanding" (and LDS reads done if LGKM0)
template <int N, bool LGKM0>
__device__ __forceinline__ void wait_vm() {
  constexpr int imm = (N & 15) | ((N >> 4) << 14) | (7 << 4) | ((LGKM0 ? 0 : 15) << 8);
  __builtin_amdgcn_s_waitcnt(imm);
  asm volatile("" ::: "memory");
}

// Workgroup barrier without the memory fence of __syncthreads(): the callers wait for exactly the
// loads and LDS reads they need (wait_vm) just before it; a fence would make the compiler wait for
// EVERY slab still in flight.
__device__ __forceinline__ void wg_barrier() {
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// 16 bytes per lane from global memory straight into LDS through a buffer descriptor: address =
// base + voff (per lane) + soff (wave-uniform), all in bytes; the descriptor (raw buffer, no bounds
// in practice) is rebuilt from the base pointer at each call site and hoisted by the compiler.
__device__ __forceinline__ void buffer_load_lds16(const void* base, lptr_t dst, uint32_t voff, int soff) {
  const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void*)base, (short)0, (int)0xFFFFFFFFu, 0x00020000);
  __builtin_amdgcn_raw_ptr_buffer_load_lds(r, dst, 16, voff, soff, 0, 0);
}

// tile t of a problem -> (tile row, tile column): groups of 8 tile rows, column-major inside
__device__ __forceinline__ void tile_coords(const GemmProblem& P, int t, int& tm, int& tn) {
  constexpr int GM = 8;
  int per = GM * P.tiles_n;
  int g = t / per, r = t - g * per;
  int first = g * GM;
  int gsz = P.tiles_m - first < GM ? P.tiles_m - first : GM;
  tm = first + r % gsz;
  tn = r / gsz;
}

// MODE: 0 = production; 4 = split-K: workgroup b = tile*splits + s walks the s-th share of the
// k-slabs and leaves its fp32 accumulators, in register order, in chunk b of batch.partial for
// splitk_reduce_kernel (small-M problems have too few tiles to fill the chip and a lone
// tile's k-loop runs at global-memory latency per slab).
// CONV: every problem of the batch is a 3x3 convolution (GemmProblem::conv_w > 0); a separate
// instantiation so that the plain product's address arithmetic stays as it is.
// Slabs are fetched with buffer_load ... lds: descriptor in SGPRs, one 32-bit byte offset per lane, taken
// from the tile's first row (for a convolution: from that row's window) and never changing, the k advance
// in an SGPR: no vector address arithmetic in the loop and a cheaper issue than global_load_lds with
// 64-bit lane addresses (measured +2..7 %, convolutions +2.5 %).
// SCHED: how the loop is laid out.
//   2  k-steps of a slab in order, the barrier after the last fragment read
//   3  the loop rotated: an iteration starts right after the barrier with the LAST k-step of a
//      slab, so its first MFMAs wait for no LDS read (measured 0..+3 % on the 8-wave 256x256 tile, not on
//      the 4-wave 128x128 one)
template <int BM, int BN, int WM, int WN, int BKT, int NS, int MODE, bool CONV = false, int SCHED = 2>
__global__ __launch_bounds__(WM * WN * 64) void gemm_kernel(const GemmBatch batch) {
  constexpr int NT = WM * WN * 64;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr int ROWB = BKT * 2;                        // bytes of one slab row in LDS
  constexpr int CPR = BKT / 8;                         // 16-byte chunks per slab row
  constexpr int KK = BKT / 16;                         // k-steps per slab (2 or 4)
  constexpr int LA = BM * CPR / NT, LB = BN * CPR / NT;   // chunks per thread per slab
  constexpr int LPS = LA + LB;
  static_assert(BM * CPR % NT == 0 && BN * CPR % NT == 0, "tile/threads");
  static_assert((NS - 1) * LPS < 64, "vmcnt range");
  extern __shared__ __attribute__((aligned(128))) unsigned char smem[];
  constexpr int STAGE = (BM + BN) * ROWB;   // one slab of A then one slab of W
  constexpr int OFFB = BM * ROWB;

  // ---- workgroup -> (problem, tile) ----------------------------------------------------
  int bid = blockIdx.x, nb = gridDim.x;
  {
    int x = bid & 7, idx = bid >> 3, q = nb >> 3, rem = nb & 7;
    bid = x * q + (x < rem ? x : rem) + idx;
  }
  const int chunk = bid;          // split-K: this workgroup's slot in batch.partial
  int split = 0;
  if (MODE == 4) { split = bid % batch.splits; bid /= batch.splits; }
  GemmProblem P = batch.p[0];   // static indices only: keeps the argument block in SGPRs
  if (batch.n > 1 && bid >= batch.p[1].tile_start) P = batch.p[1];
  if (batch.n > 2 && bid >= batch.p[2].tile_start) P = batch.p[2];
  int tm, tn;
  tile_coords(P, bid - P.tile_start, tm, tn);
  const int m0 = tm * BM, n0 = tn * BN;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;

  // ---- per-thread global source offsets ------------------------------------------------
  // (element offsets from the matrix base; every operand is far below 2^31 elements)
  uint32_t ga[LA], gb[LB];
  size_t conv_pix0 = 0;        // convolution: window of row m0 in the stack of bordered images
  if constexpr (CONV) {
    const int mm = m0 < P.M ? m0 : P.M - 1;
    const int b = mm / P.conv_img, r = mm - b * P.conv_img;
    const int y = r / P.conv_w, x = r - y * P.conv_w;
    conv_pix0 = (size_t)(b * (P.conv_img / P.conv_w + 2) + y) * (P.conv_w + 2) + x;
  }
#pragma unroll
  for (int i = 0; i < LA; ++i) {
    int q = i * NT + tid, r = q / CPR, pc = q % CPR, c = pc ^ swz_key<BKT>(r);
    int m = m0 + r; if (m >= P.M) m = P.M - 1;            // clamp: rows past M are never stored
    if constexpr (CONV) {    // top-left pixel of the 3x3 window in the stack of bordered images
      const int b = m / P.conv_img, r = m - b * P.conv_img;
      const int y = r / P.conv_w, x = r - y * P.conv_w;
      const size_t pix = (size_t)(b * (P.conv_img / P.conv_w + 2) + y) * (P.conv_w + 2) + x;
      // from the window of the tile's first row (pixels of later rows lie behind it)
      ga[i] = (uint32_t)((pix - conv_pix0) * (size_t)P.conv_cin) + c * 8;
    } else {
      ga[i] = (uint32_t)(m - m0) * (uint32_t)P.lda + c * 8;    // from the tile's first row (the buffer's base)
    }
  }
#pragma unroll
  for (int i = 0; i < LB; ++i) {
    int q = i * NT + tid, r = q / CPR, pc = q % CPR, c = pc ^ swz_key<BKT>(r);
    gb[i] = (uint32_t)r * (uint32_t)P.ldw + c * 8; // weights are padded to N_pad rows
  }


  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  int nk = P.K / BKT;
  if (MODE == 4) {              // my share of the slabs (shares differ by at most one slab)
    const int kb = split * nk / batch.splits, ke = (split + 1) * nk / batch.splits;
    P.A += kb * BKT; P.W += kb * BKT;
    nk = ke - kb;
  }
  // lanes address their tile by 32-bit byte offsets from its first row, so no operand size limit
  const bf16_t* const tileA = CONV ? P.A + conv_pix0 * (size_t)P.conv_cin : P.A + (size_t)m0 * P.lda;
  const bf16_t* const tileW = P.W + (size_t)n0 * P.ldw;
  const int half = lane >> 5;
  // LDS byte offsets of this lane's fragment rows (the chunk index is XORed in per k-step;
  // the key is the same for rows 32 apart)
  const int arow = wm * (BM / WM) + (lane & 31);
  const int brow = wn * (BN / WN) + (lane & 31);
  const int akey = swz_key<BKT>(arow), bkey = swz_key<BKT>(brow);
  const int abase = arow * ROWB, bbase = OFFB + brow * ROWB;

  // chunk q = i*NT + tid lands at LDS byte q*16 = (i*NT + wave*64)*16 + lane*16.  Slab indices
  // past the end are clamped (the copy is redundant but keeps the load count per slab fixed,
  // which the vmcnt arithmetic below relies on).
  auto issue = [&](int kt) {
    unsigned char* dA = smem + (kt % NS) * STAGE;
    const int ks = (kt < nk ? kt : nk - 1) * BKT;
    int ka = ks;             // A-side offset of the slab
    if constexpr (CONV) {    // slab = 64 channels of one tap (ky, kx): shift by ky rows and kx pixels
      int tap = ks / P.conv_cin;
      const int c0 = ks - tap * P.conv_cin;
      int kf = 0;            // 27 taps: the first index is the frame, 0 = two frames back (the stack starts two frames early)
      if (P.conv_kt == 3) { kf = tap / 9; tap -= 9 * kf; }
      const int ky = tap / 3, kx = tap - 3 * ky;
      ka = ((kf * (P.conv_img / P.conv_w + 2) + ky) * (P.conv_w + 2) + kx) * P.conv_cin + c0;
    }
    unsigned char* dB = dA + OFFB;
#pragma unroll
    for (int i = 0; i < LA; ++i) buffer_load_lds16(tileA, (lptr_t)(dA + (i * NT + wave * 64) * 16), ga[i] * 2u, ka * 2);
#pragma unroll
    for (int i = 0; i < LB; ++i) buffer_load_lds16(tileW, (lptr_t)(dB + (i * NT + wave * 64) * 16), gb[i] * 2u, ks * 2);
  };
  auto load_frags = [&](const unsigned char* st, int kk, bf16x8 (&a)[TM], bf16x8 (&b)[TN]) {
    const int c = kk * 2 + half;
    const unsigned char* pa = st + abase + ((c ^ akey) << 4);
    const unsigned char* pb = st + bbase + ((c ^ bkey) << 4);
#pragma unroll
    for (int i = 0; i < TM; ++i) a[i] = *(const bf16x8*)(pa + i * 32 * ROWB);
#pragma unroll
    for (int j = 0; j < TN; ++j) b[j] = *(const bf16x8*)(pb + j * 32 * ROWB);
  };
  auto mfma_all = [&](const bf16x8 (&a)[TM], const bf16x8 (&b)[TN]) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  };

  bf16x8 a0[TM], b0[TN], a1[TM], b1[TN];
#pragma unroll
  for (int sidx = 0; sidx < NS; ++sidx) issue(sidx);
  wait_vm<(NS - 1) * LPS, false>();          // slab 0 has landed (mine)
  wg_barrier();   // ... and everyone's
  load_frags(smem, 0, a0, b0);
  if constexpr (SCHED == 3) {
    // Rotated loop: an iteration starts right after the barrier (nothing outstanding on LDS, so its first
    // MFMAs wait for nothing) with the LAST k-step of slab kt, then runs all but the last k-step of slab kt+1.
    auto front = [&](const unsigned char* cur) {       // k-steps 0 .. KK-2 of the slab in `cur`; leaves its last fragments in a1/b1
      load_frags(cur, 1, a1, b1);
      mfma_all(a0, b0);
      interleave_hint<TM + TN, TM * TN>();
      if (KK == 4) {
        load_frags(cur, 2, a0, b0);
        mfma_all(a1, b1);
        interleave_hint<TM + TN, TM * TN>();
        load_frags(cur, 3, a1, b1);
        mfma_all(a0, b0);
        interleave_hint<TM + TN, TM * TN>();
      }
    };
    front(smem);
    wait_vm<(NS - 2) * LPS, true>();         // slab 1 (mine) and my last fragments of slab 0
    wg_barrier();
    int st_cur = 0;
    for (int kt = 0; kt < nk - 1; ++kt) {
      const int st_nxt = st_cur + 1 == NS ? 0 : st_cur + 1;
      const unsigned char* nxt = smem + st_nxt * STAGE;
      issue(kt + NS);                        // into the stage of slab kt: every wave holds its last fragments
      load_frags(nxt, 0, a0, b0);
      mfma_all(a1, b1);
      interleave_hint<TM + TN, TM * TN>();
      front(nxt);
      wait_vm<(NS - 2) * LPS, true>();       // slab kt+2 (mine) has landed; my fragments are in registers
      wg_barrier();
      st_cur = st_nxt;
    }
    mfma_all(a1, b1);                        // last k-step of the last slab
  } else {
  int st_cur = 0;                            // stage of slab kt
  for (int kt = 0; kt < nk; ++kt) {
    const unsigned char* cur = smem + st_cur * STAGE;
    const int st_nxt = st_cur + 1 == NS ? 0 : st_cur + 1;
    const unsigned char* nxt = smem + st_nxt * STAGE;
    load_frags(cur, 1, a1, b1);
    mfma_all(a0, b0);
    interleave_hint<TM + TN, TM * TN>();
    if (KK == 4) {
      load_frags(cur, 2, a0, b0);
      mfma_all(a1, b1);
      interleave_hint<TM + TN, TM * TN>();
      load_frags(cur, 3, a1, b1);
      mfma_all(a0, b0);
      interleave_hint<TM + TN, TM * TN>();
    }
    // The last fragments of this slab are on their way to registers; slabs kt+1..kt+NS-1 are in
    // flight.  Wait for slab kt+1 (mine) and my fragments; after the barrier nobody reads `cur`
    // any more and `nxt` is visible to all.
    wait_vm<(NS - 2) * LPS, true>();
    wg_barrier();
    issue(kt + NS);                          // into the stage of slab kt
    load_frags(nxt, 0, a0, b0);              // (after the last slab this reads a stale stage; unused)
    mfma_all(a1, b1);
    interleave_hint<TM + TN, TM * TN>();
    st_cur = st_nxt;
  }
  }
  wait_vm<0, true>();                        // drain the redundant tail loads before LDS is released
  if (MODE == 4) {
    // float4 number q = (((wave*TM + i)*TN + j)*4 + g)*64 + lane of the chunk holds
    // C[32i + 8g + 4*half + 0..3][32j + lane%32] of wave's sub-tile: 1 KB per store instruction
    float* pc = batch.partial + (size_t)chunk * (BM * BN);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          f32x4 v4 = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
          *(f32x4*)(pc + ((((wave * TM + i) * TN + j) * 4 + g) * 64 + lane) * 4) = v4;
        }
    return;
  }

  // ---- epilogue ---------------------------------------------------------------------------
  // acc[i][j][e] is C[32i + 8*(e/4) + 4*half + e%4][32j + lane%32] of the wave's sub-tile: a lane
  // holds one column, so direct stores would be 2- or 4-byte pieces.  Each wave therefore turns
  // its sub-tile 32 rows at a time through a private LDS patch (row stride TN*128 + 32 bytes:
  // the two half-waves, 4 rows apart, then fall into disjoint bank halves) and reads it back
  // row-major, 4 (fp32 out) or 8 (bf16 out) consecutive columns per lane: global accesses are
  // 16 bytes per lane and whole rows of the sub-tile per instruction.
  __syncthreads();     // every wave's ring loads have landed and all fragment reads are done
  constexpr int RS = TN * 128 + 32;
  unsigned char* stg = smem + wave * (32 * RS);
  static_assert(WM * WN * 32 * RS <= NS * STAGE, "staging patch fits the ring");
  auto epilogue = [&](auto kind_tag) {
    constexpr int KIND = decltype(kind_tag)::value;
    constexpr bool F32OUT = KIND == OUT_F32 || KIND == OUT_RESID_F32;
    constexpr int VEC = F32OUT ? 4 : 8;          // columns per lane
    constexpr int LPR = TN * 32 / VEC;           // lanes per row
    constexpr int RPI = 64 / LPR;                // rows per instruction
    const int lr = lane / LPR, lc = (lane % LPR) * VEC;
    const int n = n0 + wn * (BN / WN) + lc;      // first of this lane's columns
    const bool full = n + VEC <= P.N;
    float bv[VEC];
#pragma unroll
    for (int c = 0; c < VEC; ++c) bv[c] = (P.bias && n + c < P.N) ? P.bias[n + c] : 0.f;
    // convolutions with fp32 output: per-column sums and sums of squares of the values stored,
    // over this wave's rows (the statistics pass of the group norm that follows)
    constexpr bool STATS = CONV && F32OUT;
    float cs[STATS ? VEC : 1], cq[STATS ? VEC : 1];
    if constexpr (STATS) {
#pragma unroll
      for (int c = 0; c < VEC; ++c) { cs[c] = 0.f; cq[c] = 0.f; }
    }
    // Gated residual: the loads of an output row (request index -> gate vector, and the residual itself)
    // depend on each other and may not be moved across the stores by the compiler, so they are issued
    // by hand for all rows of a 32-row patch at once: two memory latencies per patch instead of two per row.
    constexpr int NIT = 32 / RPI;
    constexpr bool RESID = KIND == OUT_RESID_F32;
    int rq[RESID ? NIT : 1];
    auto load_rq = [&](int i) {
      if constexpr (RESID) {
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
          const int m = m0 + wm * (BM / WM) + i * 32 + it * RPI + lr;
          rq[it] = (P.row_req && m < P.M) ? P.row_req[m] : 0;
        }
      }
    };
    load_rq(0);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          *(float*)(stg + (8 * (e >> 2) + 4 * half + (e & 3)) * RS + (j * 32 + (lane & 31)) * 4) = acc[i][j][e];
      f32x4 xr[RESID ? NIT : 1], gr[RESID ? NIT : 1];
      // (tiles with 128 or more accumulator registers per lane fetch half a patch at a time)
      constexpr int GRP = (RESID && TM * TN >= 8) ? NIT / 2 : NIT;
      auto load_resid = [&](int first) {
        if constexpr (RESID) {
#pragma unroll
          for (int it = first; it < first + GRP; ++it) {
            const int m = m0 + wm * (BM / WM) + i * 32 + it * RPI + lr;
            xr[it] = f32x4{0.f, 0.f, 0.f, 0.f};
            gr[it] = f32x4{1.f, 1.f, 1.f, 1.f};
            if (full && m < P.M) {
              xr[it] = *(const f32x4*)((const float*)P.out + (size_t)m * P.ldc + n);
              if (P.gate) gr[it] = *(const f32x4*)(P.gate + (size_t)rq[it] * P.gate_stride + n);
            }
          }
        }
      };
      load_resid(0);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        if (GRP < NIT && it == GRP) load_resid(GRP);
        if (RESID && it == NIT - 1 && i + 1 < TM) load_rq(i + 1);
        const int row = it * RPI + lr;
        const int m = m0 + wm * (BM / WM) + i * 32 + row;
        float v[VEC];
#pragma unroll
        for (int c4 = 0; c4 < VEC / 4; ++c4) {
          const f32x4 t4 = *(const f32x4*)(stg + row * RS + (lc + 4 * c4) * 4);
#pragma unroll
          for (int c = 0; c < 4; ++c) v[4 * c4 + c] = t4[c] + bv[4 * c4 + c];
        }
        if (m >= P.M || n >= P.N) continue;
        const size_t o = (size_t)m * P.ldc + n;
        if constexpr (KIND == OUT_RESID_F32) {
          float* xp = (float*)P.out + o;
          if (full) {
            f32x4 x4 = xr[it];
#pragma unroll
            for (int c = 0; c < 4; ++c) x4[c] += gr[it][c] * v[c];
            *(f32x4*)xp = x4;
            if constexpr (STATS) {
#pragma unroll
              for (int c = 0; c < 4; ++c) { cs[c] += x4[c]; cq[c] += x4[c] * x4[c]; }
            }
          } else {
            // (ragged last columns: the request index is read here, rq[] may already hold the next patch's)
            const float* gp = P.gate ? P.gate + (size_t)(P.row_req ? P.row_req[m] : 0) * P.gate_stride + n : nullptr;
            for (int c = 0; c < VEC && n + c < P.N; ++c) {
              const float r = xp[c] + (gp ? gp[c] : 1.f) * v[c];
              xp[c] = r;
              if constexpr (STATS) { cs[c] += r; cq[c] += r * r; }
            }
          }
        } else if constexpr (KIND == OUT_F32) {
          float* xp = (float*)P.out + o;
          if (full) {
            f32x4 x4 = {v[0], v[1], v[2], v[3]};
            *(f32x4*)xp = x4;
          } else {
            for (int c = 0; c < VEC && n + c < P.N; ++c) xp[c] = v[c];
          }
          if constexpr (STATS) {
#pragma unroll
            for (int c = 0; c < VEC; ++c) { cs[c] += v[c]; cq[c] += v[c] * v[c]; }   // (columns past N are not written out)
          }
        } else {
          if constexpr (KIND == OUT_GELU_BF16) {
#pragma unroll
            for (int c = 0; c < VEC; ++c) v[c] = gelu_tanh(v[c]);
          }
          bf16_t* xp = (bf16_t*)P.out + o;
          if (full) {
            u32x4 w;
#pragma unroll
            for (int c = 0; c < 4; ++c) w[c] = pack2bf(v[2 * c], v[2 * c + 1]);
            *(u32x4*)xp = w;
          } else {
            for (int c = 0; c < VEC && n + c < P.N; ++c) xp[c] = f2bf(v[c]);
          }
        }
      }
      asm volatile("" ::: "memory");
    }
    if constexpr (STATS) {
      if (P.stats) {      // partial[(tile row * WM + wm)][column][2]: rows of one wave of one tile
#pragma unroll
        for (int c = 0; c < VEC; ++c)
#pragma unroll
          for (int o = LPR; o < 64; o <<= 1) { cs[c] += __shfl_xor(cs[c], o); cq[c] += __shfl_xor(cq[c], o); }
        if (lr == 0) {
          float* sp = P.stats + ((size_t)(tm * WM + wm) * P.N + n) * 2;
          for (int c = 0; c < VEC && n + c < P.N; ++c) { sp[2 * c] = cs[c]; sp[2 * c + 1] = cq[c]; }
        }
      }
    }
  };
  // q/k columns of a QKV product: RMS norm per head, gain, rotary code, scale, scatter by row.
  // A wave's 64 columns are one head (head_dim 64) or half of one (128: the two waves of a
  // pair exchange their partial sums of squares through LDS).
  auto epilogue_qk = [&]() {
    if constexpr (BN / WN == 64) {
      constexpr int VEC = 8, LPR = 8, RPI = 8;
      const QkNorm& Q = P.qk;
      const int lr = lane / LPR, lc = (lane % LPR) * VEC;
      const int n = n0 + wn * 64 + lc;               // first of this lane's 8 output columns
      const bool is_k = n >= Q.nq;
      const int col_in = is_k ? n - Q.nq : n;        // column inside the q (k) range
      const int hc = col_in & (Q.head_dim - 1);      // ... inside the head
      const bool wide = Q.head_dim == 128;
      const float inv_dh = 1.0f / (float)Q.head_dim;
      const float osc = is_k ? 1.0f : Q.qscale;
      float bv[VEC], gv[VEC];
      {
        const float* gp = (is_k ? Q.kgain : Q.qgain) + hc;
        const f32x4 g0 = *(const f32x4*)gp, g1 = *(const f32x4*)(gp + 4);
#pragma unroll
        for (int c = 0; c < 4; ++c) { gv[c] = g0[c]; gv[4 + c] = g1[c]; }
#pragma unroll
        for (int c = 0; c < VEC; ++c) bv[c] = P.bias ? P.bias[n + c] : 0.f;
      }
      float* xch = (float*)(smem + WM * WN * 32 * RS);   // [2][waves][32] partial sums of squares
      static_assert(WM * WN * 32 * RS + 2 * WM * WN * 32 * 4 <= NS * STAGE, "exchange area fits the ring");
      bf16_t* dst = is_k ? Q.ko : Q.qo;
      // Destination rows one patch ahead, and per patch the rotary pairs of its rows while the patch
      // turns through LDS: the compiler may not move these loads across the stores, and issued row by row
      // each would cost a full memory latency.
      int dnext[4];
      auto load_drows = [&](int i) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const int m = m0 + wm * (BM / WM) + i * 32 + it * RPI + lr;
          dnext[it] = (Q.dst_row && m < P.M) ? Q.dst_row[m] : m;
        }
      };
      load_drows(0);
#pragma unroll
      for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int e = 0; e < 16; ++e)
            *(float*)(stg + (8 * (e >> 2) + 4 * half + (e & 3)) * RS + (j * 32 + (lane & 31)) * 4) = acc[i][j][e];
        int drows[4];
        f32x4 rc0[4], rc1[4];
        constexpr int RG = TM * TN >= 10 ? 1 : 4;     // (the 320-row tile has no registers to spare: row by row there;
                                                      //  2 or 4 rows at a time spill and measured slower)
        auto load_rope = [&](int first) {
#pragma unroll
          for (int it = first; it < first + RG; ++it) {
            const int m = m0 + wm * (BM / WM) + i * 32 + it * RPI + lr;
            rc0[it] = f32x4{1.f, 0.f, 1.f, 0.f}; rc1[it] = f32x4{1.f, 0.f, 1.f, 0.f};      // (cos, sin) pairs
            if (Q.rope && m < P.M) {
              const f32x4* rp = (const f32x4*)(Q.rope + (size_t)drows[it] * (Q.head_dim / 2) + (hc >> 1));
              rc0[it] = rp[0]; rc1[it] = rp[1];
            }
          }
        };
#pragma unroll
        for (int it = 0; it < 4; ++it) drows[it] = dnext[it];
        load_rope(0);
        if (i + 1 < TM) load_drows(i + 1);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        float v[4][VEC], ss[4];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const int row = it * RPI + lr;
          const f32x4 t0 = *(const f32x4*)(stg + row * RS + lc * 4), t1 = *(const f32x4*)(stg + row * RS + (lc + 4) * 4);
          float s2 = 0.f;
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            v[it][c] = t0[c] + bv[c]; v[it][4 + c] = t1[c] + bv[4 + c];
            s2 += v[it][c] * v[it][c] + v[it][4 + c] * v[it][4 + c];
          }
          s2 += __shfl_xor(s2, 1); s2 += __shfl_xor(s2, 2); s2 += __shfl_xor(s2, 4);
          ss[it] = s2;
        }
        if (wide) {
          float* mine = xch + ((i & 1) * (WM * WN) + wave) * 32;
          const float* other = xch + ((i & 1) * (WM * WN) + (wave ^ 1)) * 32;
          if ((lane % LPR) == 0) {
#pragma unroll
            for (int it = 0; it < 4; ++it) mine[it * RPI + lr] = ss[it];
          }
          __syncthreads();
#pragma unroll
          for (int it = 0; it < 4; ++it) ss[it] += other[it * RPI + lr];
        }
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          if (RG < 4 && it > 0 && it % RG == 0) load_rope(it);
          const int m = m0 + wm * (BM / WM) + i * 32 + it * RPI + lr;
          if (m >= P.M) continue;
          const float r = rsqrtf(ss[it] * inv_dh + 1e-6f) * osc;
          const int drow = drows[it];
          const f32x4 c0 = rc0[it], c1 = rc1[it];
          const float cs[8] = {c0[0], c0[1], c0[2], c0[3], c1[0], c1[1], c1[2], c1[3]};
          u32x4 w;
#pragma unroll
          for (int pz = 0; pz < 4; ++pz) {
            const float a = v[it][2 * pz] * r * gv[2 * pz], b = v[it][2 * pz + 1] * r * gv[2 * pz + 1];
            const float ra = a * cs[2 * pz] - b * cs[2 * pz + 1], rb = a * cs[2 * pz + 1] + b * cs[2 * pz];
            w[pz] = Q.f16 ? pack2h(ra, rb) : pack2bf(ra, rb);
          }
          *(u32x4*)(dst + (size_t)drow * Q.ldo + col_in) = w;
        }
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);    // patches one after the other: work hoisted across them costs registers
      }
    }
  };
  // value columns of a QKV product written transposed (the layout the attention kernel reads): the
  // wave's 32-row patch goes through LDS column-major, and a lane writes two consecutive rows of one
  // output column as one 4-byte piece when they are neighbours in the transposed matrix (always, except
  // across a request boundary or at an odd start), else as single elements.
  auto epilogue_vt = [&]() {
   if constexpr (BN / WN == 64) {                      // (the tile variants that take q/k-norm problems)
    const QkNorm& Q = P.qk;
    constexpr int CS = 36 * 4;                         // bytes per patch column: 32 rows + padding, 16-byte aligned
    static_assert(TN * 32 * CS <= 32 * RS, "transposed patch fits the wave's staging area");
    const int nv0 = n0 + wn * (BN / WN) - (Q.nq + Q.nk);   // first value column of the wave
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          *(float*)(stg + (j * 32 + (lane & 31)) * CS + (8 * (e >> 2) + 4 * half + (e & 3)) * 4) = acc[i][j][e];
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      const int mb = m0 + wm * (BM / WM) + i * 32;     // first row of the patch
      // whole patch in range, its 32 rows neighbours in the transposed matrix, starting at a multiple of 8:
      // a lane writes 8 rows of one column as one 16-byte piece
      bool consec = mb + 32 <= P.M;
      int cb = 0;
      if (consec) {
        cb = Q.vt_col[mb];
        consec = Q.vt_col[mb + 31] == cb + 31;
      }
      if (consec && (cb & 7) != 0) {
        // Neighbours, but starting off a multiple of 8 (a request's image rows follow 154 text rows): three
        // 16-byte pieces from the first aligned column on, written by lanes 0-2 of each group of four; the
        // fourth lane writes the 8 rows before and after them as pairs (even start) or single elements.
        const int r0 = 8 - (cb & 7);                   // patch row of the first aligned column
        const int rg = lane & 3, cl = lane >> 2;
#pragma unroll
        for (int it = 0; it < TN * 32 / 16; ++it) {
          const int col = it * 16 + cl, nv = nv0 + col;
          if (nv + Q.nq + Q.nk >= P.N) continue;
          const float* pc = (const float*)(stg + col * CS);
          const float bv = P.bias ? P.bias[nv + Q.nq + Q.nk] : 0.f;
          bf16_t* dst = Q.vt + (size_t)nv * Q.ldvt + cb;
          if (rg < 3) {
            const float* t = pc + r0 + 8 * rg;
            u32x4 w = {pack2bf(t[0] + bv, t[1] + bv), pack2bf(t[2] + bv, t[3] + bv), pack2bf(t[4] + bv, t[5] + bv), pack2bf(t[6] + bv, t[7] + bv)};
            *(u32x4*)(dst + r0 + 8 * rg) = w;
          } else if ((cb & 1) == 0) {
#pragma unroll
            for (int k = 0; k < 8; k += 2) {
              const int r = k < r0 ? k : k + 24;
              *(uint32_t*)(dst + r) = pack2bf(pc[r] + bv, pc[r + 1] + bv);
            }
          } else {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
              const int r = k < r0 ? k : k + 24;
              dst[r] = f2bf(pc[r] + bv);
            }
          }
        }
      } else if (consec) {
        const int rg = lane & 3, cl = lane >> 2;
#pragma unroll
        for (int it = 0; it < TN * 32 / 16; ++it) {
          const int col = it * 16 + cl, nv = nv0 + col;
          const f32x4 t0 = *(const f32x4*)(stg + col * CS + rg * 32), t1 = *(const f32x4*)(stg + col * CS + rg * 32 + 16);
          if (nv + Q.nq + Q.nk >= P.N) continue;
          const float bv = P.bias ? P.bias[nv + Q.nq + Q.nk] : 0.f;
          u32x4 w = {pack2bf(t0[0] + bv, t0[1] + bv), pack2bf(t0[2] + bv, t0[3] + bv), pack2bf(t1[0] + bv, t1[1] + bv), pack2bf(t1[2] + bv, t1[3] + bv)};
          *(u32x4*)(Q.vt + (size_t)nv * Q.ldvt + cb + rg * 8) = w;
        }
      } else {
        const int rp = lane & 15, cl = lane >> 4;      // this lane's row pair and column phase
        const int m = mb + 2 * rp;
        const bool ok0 = m < P.M, ok1 = m + 1 < P.M;
        const int c0 = ok0 ? Q.vt_col[m] : 0, c1 = ok1 ? Q.vt_col[m + 1] : -1;
        const bool pair = ok1 && c1 == c0 + 1 && (c0 & 1) == 0;
#pragma unroll
        for (int it = 0; it < TN * 32 / 4; ++it) {
          const int col = it * 4 + cl;                 // column inside the wave's patch
          const int nv = nv0 + col;                    // value column = row of the transposed matrix
          const f32x2 t2 = *(const f32x2*)(stg + col * CS + rp * 8);
          if (nv + Q.nq + Q.nk >= P.N) continue;
          const float bv = P.bias ? P.bias[nv + Q.nq + Q.nk] : 0.f;
          bf16_t* dst = Q.vt + (size_t)nv * Q.ldvt;
          if (pair) *(uint32_t*)(dst + c0) = pack2bf(t2[0] + bv, t2[1] + bv);
          else {
            if (ok0) dst[c0] = f2bf(t2[0] + bv);
            if (ok1) dst[c1] = f2bf(t2[1] + bv);
          }
        }
      }
      asm volatile("" ::: "memory");
    }
   }
  };
  if (P.out_kind == OUT_QKNORM) {
    if (n0 < P.qk.nq + P.qk.nk) epilogue_qk();
    else if (P.qk.vt) epilogue_vt();
    else epilogue(std::integral_constant<int, OUT_BF16>{});
  }
  else if (P.out_kind == OUT_BF16) epilogue(std::integral_constant<int, OUT_BF16>{});
  else if (P.out_kind == OUT_F32) epilogue(std::integral_constant<int, OUT_F32>{});
  else if (P.out_kind == OUT_GELU_BF16) epilogue(std::integral_constant<int, OUT_GELU_BF16>{});
  else epilogue(std::integral_constant<int, OUT_RESID_F32>{});
}

// Second half of a split-K product: sums the `splits` partial tiles in fixed order (so the
// result does not depend on which workgroup finished first) and applies the epilogue.  One
// thread per float4 of the chunk layout written above: 4 consecutive rows of one column, the
// 32 lanes of a half-wave on 32 consecutive columns.
template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const GemmBatch batch) {
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr int QPT = BM * BN / 4;                 // float4s per tile
  constexpr int BPT = QPT / 256;                   // workgroups per tile
  const int tile = blockIdx.x / BPT;
  const int q = (blockIdx.x % BPT) * 256 + threadIdx.x;
  GemmProblem P = batch.p[0];
  if (batch.n > 1 && tile >= batch.p[1].tile_start) P = batch.p[1];
  if (batch.n > 2 && tile >= batch.p[2].tile_start) P = batch.p[2];
  int tm, tn;
  tile_coords(P, tile - P.tile_start, tm, tn);
  const int lane = q & 63, g = (q >> 6) & 3, j = (q >> 8) % TN, i = (q >> 8) / TN % TM, wave = (q >> 8) / (TN * TM);
  const int wm = wave / WN, wn = wave % WN;
  const int n = tn * BN + wn * (BN / WN) + j * 32 + (lane & 31);
  const int mrow = tm * BM + wm * (BM / WM) + i * 32 + 8 * g + 4 * (lane >> 5);
  const float* pc = batch.partial + (size_t)tile * batch.splits * (BM * BN) + (size_t)q * 4;
  f32x4 acc = *(const f32x4*)pc;
  for (int s = 1; s < batch.splits; ++s) {
    const f32x4 t4 = *(const f32x4*)(pc + (size_t)s * (BM * BN));
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[c] += t4[c];
  }
  if (n >= P.N) return;
  const float bias = P.bias ? P.bias[n] : 0.f;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int m = mrow + c;
    if (m >= P.M) continue;
    const float v = acc[c] + bias;
    const size_t o = (size_t)m * P.ldc + n;
    if (P.out_kind == OUT_RESID_F32) {
      const float gt = P.gate ? P.gate[(size_t)(P.row_req ? P.row_req[m] : 0) * P.gate_stride + n] : 1.f;
      ((float*)P.out)[o] += gt * v;
    } else if (P.out_kind == OUT_F32) {
      ((float*)P.out)[o] = v;
    } else {
      ((bf16_t*)P.out)[o] = f2bf(P.out_kind == OUT_GELU_BF16 ? gelu_tanh(v) : v);
    }
  }
}

template <int BM, int BN, int WM, int WN, int BKT, int NS, int MODE = 0, bool CONV = false, int SCHED = 2>
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
  size_t lds = (size_t)NS * (BM + BN) * BKT * 2;
  auto kern = gemm_kernel<BM, BN, WM, WN, BKT, NS, MODE, CONV, SCHED>;
  static std::atomic<unsigned> seen{0};
  if (first_use_on_device(seen))
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (MODE == 4) {
    hipLaunchKernelGGL(kern, dim3(total * b.splits), dim3(WM * WN * 64), lds, s, b);
    hipLaunchKernelGGL((splitk_reduce_kernel<BM, BN, WM, WN>), dim3(total * (BM * BN / 1024)), dim3(256), 0, s, b);
  } else {
    hipLaunchKernelGGL(kern, dim3(total), dim3(WM * WN * 64), lds, s, b);
  }
}

// variant codes: BM*1000 + BN, plus
//   +1000000  8 waves (2x4) instead of 4 (2x2); 1320256: 320x256 with 8 waves
//   +10000000 k-slab 32 with a 4-stage ring, +20000000 k-slab 32 with a 5-stage ring
//             (default: k-slab 64, 2 stages)
//   31256128 / 32256128 / 31128256  256x128 (4 waves / 8 waves) and 128x256 with a 3-stage ring
//   30128128  128x128, k-slab 64, 4-stage ring (one workgroup per CU: for grids below 256 tiles)
//   30128064 / 33128064  128x64 (4 waves of 32x64), 6- / 3-stage ring;  30064128  64x128 (4 waves of 64x32), 6-stage ring
//   40128128  the same as split-K over b.splits shares of K plus the reduction kernel
int launch_gemm(hipStream_t s, GemmBatch& b, int force_tile) {
  // Tile choice.  The 256x256 tile (8 waves) halves the L2->LDS traffic per flop of the 128x128
  // tile and is about 25% faster per tile-flop, but one workgroup fills a CU, so its grid runs
  // in rounds of 256 tiles: use it from one full round on, unless the last round would hold only
  // a few tiles (measured over the benchmark shapes: a partly filled last round runs faster
  // than a full one, lone tiles see less contention); otherwise the 128x128 tile (three
  // workgroups per CU, finer granularity).
  int tile = force_tile;
  if (tile == 40128128 && (!b.partial || b.splits < 1)) tile = 30128128;   // no scratch: no split
  if (tile != 40128128) b.splits = 1;
  if (!tile) {
    // Few tiles (small M): a lone tile's k-loop runs at memory latency per slab, so keep three
    // slabs in flight (4-stage ring, one workgroup per CU) and, when K is long enough, split it
    // over up to 256 workgroups.
    long long t128 = 0;
    int min_nk = 1 << 30;
    for (int i = 0; i < b.n; ++i) {
      if (b.p[i].M <= 0 || b.p[i].N <= 0) continue;
      t128 += (long long)((b.p[i].M + 127) / 128) * ((b.p[i].N + 127) / 128);
      min_nk = b.p[i].K / 64 < min_nk ? b.p[i].K / 64 : min_nk;
    }
    if (t128 > 0 && t128 <= 256) {
      long long sp = 256 / t128;
      if (sp > min_nk / 4) sp = min_nk / 4;
      const long long cap = (long long)(b.partial_bytes / (128 * 128 * 4)) / t128;
      if (sp > cap) sp = cap;
      bool qk = false;                       // the reduction kernel has no q/k-norm epilogue
      for (int i = 0; i < b.n; ++i) qk = qk || b.p[i].out_kind == OUT_QKNORM || b.p[i].conv_w > 0;   // (nor the split A offsets a convolution's)
      if (b.partial && sp >= 2 && !qk) { b.splits = (int)sp; tile = 40128128; }
      else {
        // no split (q/k-norm epilogue, or K too short): 128x64 tiles with a 6-stage ring when twice the
        // workgroups still fit one round: these launches run at memory latency, and twice as many CUs with
        // more bytes in flight each fetch the weights faster (108 -> 216 workgroups: 17.4 -> 13.2 us)
        long long t64 = 0;
        for (int i = 0; i < b.n; ++i)
          if (b.p[i].M > 0 && b.p[i].N > 0) t64 += (long long)((b.p[i].M + 127) / 128) * ((b.p[i].N + 63) / 64);
        bool narrow_ok = true;        // not for convolutions; a 128-wide head must lie inside one workgroup's columns
        for (int i = 0; i < b.n; ++i)
          narrow_ok = narrow_ok && b.p[i].conv_w <= 0 && !(b.p[i].out_kind == OUT_QKNORM && b.p[i].qk.head_dim > 64);
        tile = (t64 <= 256 && narrow_ok) ? 30128064 : 30128128;
        if (tile == 30128128 && !qk) {          // ... or 64-row tiles when that gives more workgroups in one round
          long long t6 = 0;
          bool plain = true;
          for (int i = 0; i < b.n; ++i) {
            if (b.p[i].M > 0 && b.p[i].N > 0) t6 += (long long)((b.p[i].M + 63) / 64) * ((b.p[i].N + 127) / 128);
            plain = plain && b.p[i].conv_w <= 0;
          }
          if (plain && t6 <= 256 && t6 > t128) tile = 30064128;
        }
      }
    }
  }
  if (!tile) {
    // One round of 256x128 tiles (8 waves, 3-stage ring) when that fits the chip and K is not short:
    // a workgroup per CU with three slabs in flight, against 1.6 128x128 workgroups per CU (measured on the
    // 4250-row request: 7 % faster at K = 6144, 3 % at K = 1536).
    long long t21 = 0;
    int min_k = 1 << 30;
    bool plain = true;
    for (int i = 0; i < b.n; ++i) {
      if (b.p[i].M <= 0 || b.p[i].N <= 0) continue;
      t21 += (long long)((b.p[i].M + 255) / 256) * ((b.p[i].N + 127) / 128);
      min_k = b.p[i].K < min_k ? b.p[i].K : min_k;
      plain = plain && b.p[i].out_kind != OUT_QKNORM && b.p[i].conv_w <= 0;
    }
    if (plain && t21 > 128 && t21 <= 256 && min_k >= 1536) tile = 32256128;
  }
  if (!tile) {
    int max_n = 0;
    for (int i = 0; i < b.n; ++i)
      if (b.p[i].M > 0 && b.p[i].N > max_n) max_n = b.p[i].N;
    if (max_n <= 128) tile = 128128;       // half or more of a 256-wide tile would be padding
  }
  if (!tile) {
    long long t256 = 0;
    for (int i = 0; i < b.n; ++i)
      t256 += (long long)((b.p[i].M + 255) / 256) * ((b.p[i].N + 255) / 256);
    const long long rem = t256 % 256;
    tile = (t256 >= 1024 || (t256 >= 256 && (rem == 0 || rem >= 64))) ? 1256256 : 128128;
    // Below one round of 256x256 tiles: a round of them does the work of two rounds of 128x128 pairs in about
    // 1.67 times the time of one, so the big tile wins whenever the small one needs two rounds or more of its
    // 512 slots (216 tiles of 256x256 against 864 of 128x128 at 4608 x 3072 x 15360: 350 against 410 us).
    if (tile == 128128 && t256 < 256) {
      long long t128 = 0;
      for (int i = 0; i < b.n; ++i)
        t128 += (long long)((b.p[i].M + 127) / 128) * ((b.p[i].N + 127) / 128);
      if (100 * ((t128 + 511) / 512) > 167) tile = 1256256;      // (t256 < 256: one round of the big tile)
    }
    // A 320-row tile when it saves rounds: the 4250-row QKV product of the 1024^2 request is 306 tiles of
    // 256x256 (a second round for 50 tiles) but 252 of 320x256, one round of tiles 1.25 times as long (measured
    // 56 us against 71 us with 128x128 tiles and 77 us with 256x256); 864 tiles (4 rounds) against 720 (3 rounds
    // x 1.25) measured 5 % faster.  Per unit of work the two tiles are equally fast at K <= 5120, so the rule is
    // rounds alone, with a margin.
    bool any_conv = false;                  // (convolutions have no 320-row instantiation)
    for (int i = 0; i < b.n; ++i) any_conv = any_conv || b.p[i].conv_w > 0;
    if (t256 > 256 && !any_conv) {
      long long t320 = 0;
      for (int i = 0; i < b.n; ++i)
        t320 += (long long)((b.p[i].M + 319) / 320) * ((b.p[i].N + 255) / 256);
      const long long r256 = (t256 + 255) / 256, r320 = (t320 + 255) / 256;
      if (125 * r320 <= 95 * r256) tile = 1320256;
    }
  }
  bool conv = false, plain = false, qknorm = false;
  for (int i = 0; i < b.n; ++i) {
    conv = conv || b.p[i].conv_w > 0; plain = plain || b.p[i].conv_w <= 0;
    qknorm = qknorm || b.p[i].out_kind == OUT_QKNORM;
  }
  // the q/k-norm epilogue exists only in the instantiations whose waves own 64 output columns
  if (qknorm && !(tile == 1256256 || tile == 1320256 || tile == 11256256 || tile == 21256256 || tile == 128128 || tile == 10128128 ||
                  tile == 30128128 || tile == 30128064 || tile == 33128064 || tile == 256128 || tile == 31256128 || tile == 32256128))
    return -1;
  if (qknorm && (tile == 30128064 || tile == 33128064))      // 64 columns per workgroup: heads of 64 only
    for (int i = 0; i < b.n; ++i)
      if (b.p[i].out_kind == OUT_QKNORM && b.p[i].qk.head_dim > 64) return -1;
  if (conv) {     // convolutions: never mixed with plain products, three tile shapes
    if (plain) return -1;
    for (int i = 0; i < b.n; ++i)        // whole images of whole rows
      if (b.p[i].conv_img <= 0 || b.p[i].conv_img % b.p[i].conv_w || b.p[i].M % b.p[i].conv_img ||
          (b.p[i].conv_kt != 1 && b.p[i].conv_kt != 3) || b.p[i].K != 9 * b.p[i].conv_kt * b.p[i].conv_cin) return -1;
    if (tile == 1256256) launch_t<256, 256, 2, 4, 64, 2, 0, true, 3>(s, b);
    else if (tile == 30128128) launch_t<128, 128, 2, 2, 64, 4, 0, true, 2>(s, b);
    else { tile = 128128; launch_t<128, 128, 2, 2, 64, 2, 0, true, 2>(s, b); }
    return tile;
  }
  switch (tile) {
    case 256256: launch_t<256, 256, 2, 2, 64, 2, 0, false, 2>(s, b); break;
    case 1256256: launch_t<256, 256, 2, 4, 64, 2, 0, false, 3>(s, b); break;
    case 1320256: launch_t<320, 256, 2, 4, 64, 2, 0, false, 3>(s, b); break;
    case 10256256: launch_t<256, 256, 2, 2, 32, 4, 0, false, 2>(s, b); break;
    case 11256256: launch_t<256, 256, 2, 4, 32, 4, 0, false, 2>(s, b); break;
    case 20256256: launch_t<256, 256, 2, 2, 32, 5, 0, false, 2>(s, b); break;
    case 21256256: launch_t<256, 256, 2, 4, 32, 5, 0, false, 2>(s, b); break;
    case 256128: launch_t<256, 128, 2, 2, 64, 2, 0, false, 2>(s, b); break;
    case 128256: launch_t<128, 256, 2, 2, 64, 2, 0, false, 2>(s, b); break;
    case 10128128: launch_t<128, 128, 2, 2, 32, 4, 0, false, 2>(s, b); break;
    case 30128128: launch_t<128, 128, 2, 2, 64, 4, 0, false, 2>(s, b); break;
    case 30128064: launch_t<128, 64, 4, 1, 64, 6, 0, false, 2>(s, b); break;
    case 30064128: launch_t<64, 128, 1, 4, 64, 6, 0, false, 2>(s, b); break;
    case 33128064: launch_t<128, 64, 4, 1, 64, 3, 0, false, 2>(s, b); break;
    case 31256128: launch_t<256, 128, 2, 2, 64, 3, 0, false, 2>(s, b); break;
    case 32256128: launch_t<256, 128, 4, 2, 64, 3, 0, false, 2>(s, b); break;
    case 31128256: launch_t<128, 256, 2, 2, 64, 3, 0, false, 2>(s, b); break;
    case 40128128: launch_t<128, 128, 2, 2, 64, 4, 4, false, 2>(s, b); break;
    default: tile = 128128; launch_t<128, 128, 2, 2, 64, 2, 0, false, 2>(s, b); break;
  }
  return tile;
}

}  // namespace dit
