// Flash-style attention over packed variable-length segments on the gfx950 matrix cores.
//
//   O[q] = sum_k softmax_k(Q[q].K[k] / sqrt(dh)) V[k]      per segment and head, no mask
//
// never materialising the score matrix: keys are walked in tiles of 64 with the running
// max / running sum recurrence in fp32.
//
// Work split.  A workgroup of 4 (or 8) waves owns 128 (256) consecutive queries of one (segment, head);
// each wave owns 32 of them.  K tiles [64 keys][dh] and transposed-V tiles [dh][64 keys]
// stream through double-buffered LDS tiles via direct global->LDS loads.
//
// MFMA formulation (v_mfma_f32_32x32x16_bf16, operands: A = 32 rows x 16 k, B = 16 k x 32
// cols, a lane supplies 8 consecutive k; result: lane holds column (lane & 31), register e
// holds row 8*(e/4) + 4*(lane/32) + e%4).  Scores are computed TRANSPOSED,
//   S^T[key][query] = K_tile . Q^T ,
// so a lane holds scores of ONE query for 32 of the tile's 64 keys: the row max and row sum
// are in-register reductions plus one exchange between the two half-waves, and the
// exponentiated scores are already in B-operand position for
//   O^T[d][query] += V^T_tile[d][key] . P^T[key][query].
// For that second product the 8 values a half-wave contributes per k-step must be 8
// CONSECUTIVE keys (the V^T operand is read as 16 contiguous bytes).  The MFMA result rows
// a lane holds are {0-3, 8-11, ...} + 4*half, so K rows are fed to the first product in a
// permuted order (bits 2 and 3 of the row index swapped), which makes registers 8s..8s+7
// of a half-wave hold keys 16s + 8*half + 0..7.
#include "dit_internal.h"
#include <type_traits>

namespace dit {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void* lptr_t;

static constexpr int KT = 64;     // keys per tile

// 16 bytes per lane from global memory straight into LDS through a buffer descriptor: address = base + voff
// (per lane) + soff (wave-uniform), in bytes.  Cheaper to issue than the form with a 64-bit address per lane:
// the lane offsets of a tile never change and the tile's position is a scalar.
__device__ __forceinline__ void buffer_load_lds16(const void* base, lptr_t dst, uint32_t voff, int soff) {
  const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void*)base, (short)0, (int)0xFFFFFFFFu, 0x00020000);
  __builtin_amdgcn_raw_ptr_buffer_load_lds(r, dst, 16, voff, soff, 0, 0);
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// two floats -> packed bf16 pair, round-to-nearest-even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack2bf(float a, float b) {
  f32x2 v = {a, b};
  bf16x2 r = __builtin_convertvector(v, bf16x2);
  return *(uint32_t*)&r;
}
// value of the other half-wave's lane (lane ^ 32), combined with max / add
__device__ __forceinline__ float xhalf_max(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xhalf_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// max of three.  This file is compiled with -fno-honor-nans, so fmaxf needs no NaN
// canonicalisation of its inputs and nested calls fold into v_max3_f32.  (Scores are finite:
// q and k rows are finite and keys past a segment's end are clamped copies of its last key.)
__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

// Software pipeline of one wave, iteration kt (S = scores, P = exp'd scores):
//   region B:  S(kt+1) = K(kt+1) Q^T  [MFMA]   overlapped with   P(kt) = exp2(S(kt) - m)  [VALU]
//   region C:  O += V^T(kt) P(kt)     [MFMA]   overlapped with   row max of S(kt+1)      [VALU]
// so the matrix pipe and the vector ALU of a SIMD are busy at the same time from ONE wave
// (two waves of different workgroups on a SIMD fall into lock step and do not overlap by
// themselves).  K and V^T tiles have separate double buffers: at the barrier of iteration kt
// K(kt+1) and V(kt) have landed, K(kt+2) and V(kt+1) are issued right after it.
// MODE 3: as mode 0 plus an additive bias looked up by (key position - query position) in a
// per-head table (the text encoder's relative-position bias; its scale is the caller's).
// MODE 0: scores are multiplied by log2(e)/sqrt(dh) here; 1: the query rows already carry that
// factor, so a score is the exponent itself; 2: as 1, and the caller guarantees |q.k| <= 60 for
// every query/key pair.  In mode 2 no running max is
// kept at all: softmax is a ratio, exp2 of a bounded exponent cannot overflow fp32 or bf16
// (2^60 per term, at most 2^20 terms), and floating point keeps the same relative precision
// at any magnitude.  That path saves the subtraction, the row max and the rescale test: about
// 50 of the ~125 vector instructions per key tile, which on this machine add to, rather than
// hide under, the matrix instructions.  (q/k RMS-normalised per head, as in all three block
// families, gives |q.k| log2(e)/sqrt(dh) <= 1.44 sqrt(dh) |g_q| |g_k|: 11.5 or 16.3 for unit gains.)
// MODE 4 (cross-attention to a short condition, whose output enters the residual stream without a
// gate): as mode 1, with q and k stored as fp16 (both are RMS-normalised, hence bounded; three more
// mantissa bits in the scores) and the values as two bf16 terms, V = vt + vt_lo, both multiplied by
// the same probabilities: the rounding of k and v no longer shows in the output.
template <int DH, int NW, int MODE>
// Workgroups per CU: 4 waves at head size 64 fit 168 registers, so three workgroups share a CU (three waves per
// SIMD overlap their exponentials and matrix instructions better than two: +8 % at 4250 tokens); head size 128
// needs ~230 registers: two workgroups of 4 waves, or one of 8.
__global__ __launch_bounds__(NW * 64, NW == 4 ? (DH == 64 ? 3 : 2) : 1) void attn_kernel(const AttnArgs a) {
  constexpr int NT = NW * 64;
  constexpr int KROW = DH * 2;                 // bytes per K-tile row
  constexpr int KCPR = DH / 8;                 // 16-byte chunks per K-tile row
  constexpr int KBYTES = KT * KROW;            // K tile
  constexpr int VBYTES = DH * 128;             // V^T tile: DH rows of 64 keys
  constexpr int LK = KT * KCPR / NT;          // chunks per thread, K tile
  constexpr int LV = DH * 8 / NT;             // chunks per thread, V^T tile
  constexpr int ND = DH / 32;                  // output d-tiles
  constexpr int NKK = DH / 16;                 // k-steps of the score product
  extern __shared__ __attribute__((aligned(128))) unsigned char smem[];
  unsigned char* const sKb = smem;                   // two K tiles
  unsigned char* const sVb = smem + 2 * KBYTES;      // two V^T tiles
  unsigned char* const sVlo = smem + 2 * KBYTES + 2 * VBYTES;   // MODE 4: two tiles of the values' second term

  // ---- which (tile, head) ------------------------------------------------------------
  int bid = blockIdx.x;
  {
    int nb = gridDim.x, x = bid & 7, idx = bid >> 3, q = nb >> 3, rem = nb & 7;
    bid = x * q + (x < rem ? x : rem) + idx;
  }
  int head = bid / a.n_tiles, tidx = bid - head * a.n_tiles;
  if (a.hpx > 0) {                // tile-major inside the head group of this XCD
    const int per = a.n_tiles * a.hpx, grp = bid / per, idx = bid - grp * per;
    tidx = idx / a.hpx;
    head = grp * a.hpx + (idx - tidx * a.hpx);
  }
  const AttnTile tile = a.tiles[tidx];
  const int seg = tile.seg;
  const int qbeg = a.cu_q[seg], qlen = a.cu_q[seg + 1] - qbeg;
  const int kbeg = a.cu_k[seg], klen = a.cu_k[seg + 1] - kbeg;
  const int vcol0 = a.vt_off[seg];
  const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  // ---- Q fragments (B operand of the score product), kept in registers ---------------
  int qi = tile.q0 + wave * 32 + l32;
  const bool q_ok = qi < qlen;
  if (!q_ok) qi = qlen - 1;
  const bf16_t* qptr = a.q + (size_t)(qbeg + qi) * a.ldq + head * DH + 8 * half;
  bf16x8 qf[NKK];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) qf[kk] = *(const bf16x8*)(qptr + kk * 16);

  // ---- global -> LDS tile loads -------------------------------------------------------
  uint32_t gk[LK], gv[LV];      // element offsets
  int krow[LK];
#pragma unroll
  for (int i = 0; i < LK; ++i) {
    int q = i * NT + tid, r = q / KCPR, pc = q % KCPR;
    int c = (DH == 64) ? (pc ^ ((r >> 1) & 7)) : (pc ^ (r & 15));
    krow[i] = r;
    gk[i] = head * DH + c * 8;
  }
#pragma unroll
  for (int i = 0; i < LV; ++i) {
    int q = i * NT + tid, r = q >> 3, pc = q & 7, c = pc ^ ((r >> 1) & 7);
    gv[i] = (uint32_t)r * (uint32_t)a.ldvt + c * 8;       // from the head's first row and the segment's first column
  }
  const int n_kt_all = (klen + KT - 1) / KT;
  const int kt_first = tile.parts > 0 ? tile.kt0 : 0;                       // this workgroup's share of the key tiles
  const int n_kt = tile.parts > 0 ? tile.kt0 + tile.nkt : n_kt_all;         // (one past its last tile)
  // K tile kt: the descriptor starts at the tile's first key (no 32-bit limit on the matrix), lanes add their row
  // and chunk; V^T tile kt: one descriptor for the head's rows, the tile's first column as the scalar offset
  // (a head's DH rows of ldvt columns stay far below 4 GiB).
  const bf16_t* const kseg = a.k + (size_t)kbeg * a.ldk;
  const bf16_t* const vhead = a.vt + (size_t)head * DH * a.ldvt + vcol0;
  auto issue_k = [&](int kt) {
    unsigned char* dst = sKb + (kt & 1) * KBYTES;
    kt = kt < n_kt ? kt : n_kt - 1;
    const bf16_t* tile0 = kseg + (size_t)kt * KT * a.ldk;
    const int last = klen - 1 - kt * KT;        // rows past it are clamped copies, masked below
#pragma unroll
    for (int i = 0; i < LK; ++i) {
      const int r = krow[i] < last ? krow[i] : last;
      buffer_load_lds16(tile0, (lptr_t)(dst + (i * NT + wave * 64) * 16), ((uint32_t)r * (uint32_t)a.ldk + gk[i]) * 2u, 0);
    }
  };
  auto issue_v = [&](int kt) {
    unsigned char* dst = sVb + (kt & 1) * VBYTES;
    const int ktv = kt < n_kt ? kt : n_kt - 1;
#pragma unroll
    for (int i = 0; i < LV; ++i)
      buffer_load_lds16(vhead, (lptr_t)(dst + (i * NT + wave * 64) * 16), gv[i] * 2u, ktv * KT * 2);
    if constexpr (MODE == 4) {
      unsigned char* dlo = sVlo + (kt & 1) * VBYTES;
      const bf16_t* vlo = a.vt_lo + (size_t)head * DH * a.ldvt + vcol0;
#pragma unroll
      for (int i = 0; i < LV; ++i)
        buffer_load_lds16(vlo, (lptr_t)(dlo + (i * NT + wave * 64) * 16), gv[i] * 2u, ktv * KT * 2);
    }
  };

  // ---- LDS read offsets ------------------------------------------------------------------
  // K operand row rho = l32 reads key kappa(rho): bits 2 and 3 swapped.
  const int kap = (l32 & ~12) | ((l32 & 8) >> 1) | ((l32 & 4) << 1);
  const int kkey0 = (DH == 64) ? ((kap >> 1) & 7) : (kap & 15);   // (+32 rows does not change it)
  const int vkey = (l32 >> 1) & 7;                                 // (+32 rows does not change it)
  const int koff = kap * KROW, voff = l32 * 128;

  // S^T tile pair of key tile kt from its K buffer
  auto scores = [&](int kt, f32x16 (&st)[2]) {
    const unsigned char* sK = sKb + (kt & 1) * KBYTES + koff;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) st[t][e] = 0.f;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
      const int c = kk * 2 + half;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        bf16x8 kf = *(const bf16x8*)(sK + t * 32 * KROW + ((c ^ kkey0) << 4));
        if constexpr (MODE == 4)       // the same 16-bit containers hold fp16 values
          st[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(*(const f16x8*)&kf, *(const f16x8*)&qf[kk], st[t], 0, 0, 0);
        else
          st[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], st[t], 0, 0, 0);
      }
    }
    if constexpr (MODE == 3) {
      // additive bias by relative position (key - query), read from the per-head table.
      // Register e of tile t holds key  kt*64 + 32t + 16*(e/8) + 8*half + e%8.
      const float* bh = a.bias + (size_t)head * (2 * a.bias_L - 1);
      const int top = 2 * a.bias_L - 2;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int key = kt * KT + 32 * t + 16 * (e >> 3) + 8 * half + (e & 7);
          int idx = key - qi + a.bias_L - 1;
          idx = idx < 0 ? 0 : (idx > top ? top : idx);     // keys past the end are clamped copies, masked later
          st[t][e] += bh[idx];
        }
    }
  };
  auto row_max = [&](const f32x16 (&st)[2]) {      // four independent chains, then combined
    float m0 = max3(st[0][0], st[0][1], st[0][2]), m1 = max3(st[0][8], st[0][9], st[0][10]);
    float m2 = max3(st[1][0], st[1][1], st[1][2]), m3 = max3(st[1][8], st[1][9], st[1][10]);
    m0 = max3(m0, st[0][3], st[0][4]); m1 = max3(m1, st[0][11], st[0][12]);
    m2 = max3(m2, st[1][3], st[1][4]); m3 = max3(m3, st[1][11], st[1][12]);
    m0 = max3(m0, st[0][5], st[0][6]); m1 = max3(m1, st[0][13], st[0][14]);
    m2 = max3(m2, st[1][5], st[1][6]); m3 = max3(m3, st[1][13], st[1][14]);
    m0 = max3(m0, st[0][7], m1); m2 = max3(m2, st[1][7], m3);
    return xhalf_max(max3(m0, m2, fmaxf(st[0][15], st[1][15])));
  };

  f32x16 o[ND];
#pragma unroll
  for (int d = 0; d < ND; ++d)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[d][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c2_arg = a.scale_log2;
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};

  // ---- prologue: scores of tile 0 --------------------------------------------------------
  issue_k(kt_first);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (kt_first + 1 < n_kt) issue_k(kt_first + 1);
  issue_v(kt_first);
  f32x16 sc[2], sn[2];     // score tiles of the current and the next key tile
  scores(kt_first, sc);
  float mx = row_max(sc);

  // One iteration; `sc` holds S(kt) on entry, `sn` receives S(kt+1).  The loop below calls it
  // with the two register sets swapped on alternate tiles instead of copying sn to sc.
  auto step = [&](int kt, f32x16 (&sc)[2], f32x16 (&sn)[2]) {
    const float c2 = (MODE == 0 || MODE == 3) ? c2_arg : 1.0f;
    constexpr bool PRESCALED = MODE == 1 || MODE == 4;
    // ---- (A) raise the running max only when a row's tile max exceeds it by more than 2^8
    // in the exponent (softmax is shift-invariant, so a stale max is exact as long as nothing
    // overflows: probabilities stay below 2^8); this skips the rescale of O on most tiles.
    float mc = 0.f;
    if constexpr (MODE != 2) {
      if (__builtin_amdgcn_ballot_w64((mx - m_run) * c2 > 8.0f) != 0) {
        const float m_new = fmaxf(m_run, mx);
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c2);
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int d = 0; d < ND; ++d)
#pragma unroll
          for (int e = 0; e < 16; ++e) o[d][e] *= alpha;
      }
      mc = m_run * c2;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // my parts of K(kt+1), V(kt) have landed
    __syncthreads();                                   // everyone's; K(kt) and V(kt-1) are free
    // Head size 128: unconditional (past the last tile a redundant copy of it into a free buffer), which keeps
    // branches out of the loop body: +1.1 % at 32760 tokens; at head size 64 the branches measure 1.1 % better.
    if (DH == 128 || kt + 2 < n_kt) issue_k(kt + 2);
    if (DH == 128 || kt + 1 < n_kt) issue_v(kt + 1);

    // ---- (B) S(kt+1) on the matrix pipe while P(kt) is exponentiated on the vector ALU.
    // (After the last tile this multiplies a stale K buffer; the result is not used.  Nothing
    // between here and the end of (C) branches, so the scheduler sees one region and is left
    // to interleave the two pipes itself: explicit group hints measured 5-10% slower.)
    scores(kt + 1, sn);
    uint32_t pk[2][8];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int e = 0; e < 16; e += 2) {
        const float p0 = __builtin_amdgcn_exp2f(MODE == 2 ? sc[t][e] : PRESCALED ? sc[t][e] - mc : sc[t][e] * c2 - mc);
        const float p1 = __builtin_amdgcn_exp2f(MODE == 2 ? sc[t][e + 1] : PRESCALED ? sc[t][e + 1] - mc : sc[t][e + 1] * c2 - mc);
        const uint32_t w = pack2bf(p0, p1);
        pk[t][e >> 1] = w;
        // Row sums.  Head size 64: v_dot2_f32_bf16 on the rounded pair (one instruction per pair).  Head size 128: two
        // plain adds on the unrounded values: dot2 shares the matrix pipe and costs more beside the twice as many
        // MFMAs of this head size (+2.7 % at 32760 tokens, nothing at head size 64); these sums differ from those of
        // the rounded values by 2^-9 / sqrt(keys) relative, far below the bf16 rounding of the output.
        if constexpr (DH == 128) l_run += p0 + p1;
        else l_run = __builtin_amdgcn_fdot2_f32_bf16(*(const bf16x2*)&w, ones, l_run, false);
      }
    // ---- (C) O^T += V^T(kt) P^T(kt) on the matrix pipe while the row max of S(kt+1) is taken
    const unsigned char* sV = sVb + (kt & 1) * VBYTES + voff;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      union { uint32_t u[4]; bf16x8 v; } pf;
#pragma unroll
      for (int j = 0; j < 4; ++j) pf.u[j] = pk[s >> 1][(s & 1) * 4 + j];
      const int c = 2 * s + half;
#pragma unroll
      for (int d = 0; d < ND; ++d) {
        bf16x8 vf = *(const bf16x8*)(sV + d * 32 * 128 + ((c ^ vkey) << 4));
        o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf.v, o[d], 0, 0, 0);
        if constexpr (MODE == 4) {
          bf16x8 vl = *(const bf16x8*)(sVlo + (kt & 1) * VBYTES + voff + d * 32 * 128 + ((c ^ vkey) << 4));
          o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vl, pf.v, o[d], 0, 0, 0);
        }
      }
    }
    if constexpr (MODE != 2) mx = row_max(sn);
  };
  for (int kt = kt_first; kt < n_kt; kt += 2) {
    step(kt, sc, sn);
    if (kt + 1 < n_kt) step(kt + 1, sn, sc);
  }
  // Keys past the end of the segment in the last tile are copies of the last key (clamped loads): they cannot
  // raise the max and their V^T columns are zero, so O is unaffected; only their share of the row sum has to be
  // taken out again: the same exponentials once more (rounded to bf16 where the sums are those of the rounded
  // values).  Register e of tile t holds key  kt*64 + 32t + 16*(e/8) + 8*half + e%8.
  // (Kept out of the loop body: code there, even in a branch taken once, costs the loop 1-2 %.)
  if (n_kt == n_kt_all && (klen & (KT - 1)) != 0) {
    const int kt = n_kt_all - 1;
    const bool in_sn = ((kt - kt_first) & 1) != 0;                     // the register set the last step consumed
    const float c2 = (MODE == 0 || MODE == 3) ? c2_arg : 1.0f;
    const float mc = MODE == 2 ? 0.f : m_run * c2;
    float corr = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int key = kt * KT + 32 * t + 16 * (e >> 3) + 8 * half + (e & 7);
        const float x = in_sn ? sn[t][e] : sc[t][e];
        float pl = __builtin_amdgcn_exp2f((MODE == 0 || MODE == 3) ? x * c2 - mc : x - mc);
        if constexpr (DH == 64) pl = __uint_as_float(pack2bf(pl, 0.f) << 16);
        corr += key >= klen ? pl : 0.f;
      }
    l_run -= corr;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // the redundant tail loads, before LDS is reused or released
  float l_tot = xhalf_sum(l_run);
  // ---- key-split block: leave the unnormalised sums; the last share to arrive adds them up ----
  if constexpr (MODE == 2) {
    if (tile.parts > 0) {
      constexpr int PSZ = NW * 32 * (DH + 1);          // floats per share: O^T in register order, then the row sums
      float* const base = a.part + ((size_t)(head * a.n_slots + tile.slot) * tile.parts) * PSZ;
      float* const mine = base + (size_t)tile.part * PSZ;
      // Device-scope stores and, on the other side, device-scope loads: they go through to the level all XCDs
      // share, so no cache has to be written back or invalidated as a whole (a release fence walks this XCD's
      // L2 once per share and a full fence also drops every K and V^T line it holds for the workgroups still
      // running: measured 1.5 and 1.8 times the time of the launch without shares).
      typedef float f32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
      for (int d = 0; d < ND; ++d)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x4 v4 = {o[d][4 * g], o[d][4 * g + 1], o[d][4 * g + 2], o[d][4 * g + 3]};
          float* p4 = mine + (((wave * ND + d) * 4 + g) * 64 + lane) * 4;
          asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" :: "v"(p4), "v"(v4) : "memory");
        }
      if (half == 0)
        __hip_atomic_store((unsigned*)(mine + NW * 32 * DH + wave * 32 + l32), __float_as_uint(l_tot), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // my sums have arrived before my count
      __syncthreads();                                 // (also: every wave is done with the LDS tiles)
      if (tid == 0) {
        const unsigned old = atomicAdd(a.part_cnt + head * a.n_slots + tile.slot, 1u);
        const int last = old == (unsigned)(tile.parts - 1);
        if (last) atomicExch(a.part_cnt + head * a.n_slots + tile.slot, 0u);   // ready for the next launch
        *(volatile int*)smem = last;
      }
      __syncthreads();
      if (*(volatile int*)smem == 0) return;
      // Fixed order of summation (share 0, 1, ...; my own from registers, the same values I stored): the result
      // does not depend on which share finished last.
      f32x16 mo[ND];
#pragma unroll
      for (int d = 0; d < ND; ++d) mo[d] = o[d];
      const float ml = l_tot;
      l_tot = 0.f;
#pragma unroll
      for (int d = 0; d < ND; ++d)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[d][e] = 0.f;
      for (int pt = 0; pt < tile.parts; ++pt) {
        if (pt == tile.part) {
#pragma unroll
          for (int d = 0; d < ND; ++d)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[d][e] += mo[d][e];
          l_tot += ml;
          continue;
        }
        const float* src = base + (size_t)pt * PSZ;
#pragma unroll
        for (int d = 0; d < ND; ++d)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const float* p4 = src + (((wave * ND + d) * 4 + g) * 64 + lane) * 4;
#pragma unroll
            for (int c = 0; c < 4; c += 2) {
              const unsigned long long u = __hip_atomic_load((const unsigned long long*)(p4 + c), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              o[d][4 * g + c] += __uint_as_float((unsigned)u);
              o[d][4 * g + c + 1] += __uint_as_float((unsigned)(u >> 32));
            }
          }
        l_tot += __uint_as_float(__hip_atomic_load((const unsigned*)(src + NW * 32 * DH + wave * 32 + l32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
      }
    }
  }

  // ---- normalise and store -------------------------------------------------------------------
  if (q_ok) {
    const float inv = 1.0f / l_tot;
    const int qrow = qbeg + qi;
    const int orow = a.o_row_map ? a.o_row_map[qrow] : qrow;
    bf16_t* op = a.o + (size_t)orow * a.ldo + head * DH + 4 * half;
#pragma unroll
    for (int d = 0; d < ND; ++d)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 w;
        w.x = pack2bf(o[d][4 * g] * inv, o[d][4 * g + 1] * inv);
        w.y = pack2bf(o[d][4 * g + 2] * inv, o[d][4 * g + 3] * inv);
        *(uint2*)(op + d * 32 + 8 * g) = w;
      }
  }
}

template <int DH, int NW, int MODE>
static void launch_t(hipStream_t s, const AttnArgs& a) {
  constexpr int lds = 2 * (KT * DH * 2 + DH * 128) + (MODE == 4 ? 2 * DH * 128 : 0);   // two K tiles + two V^T tiles (+ two of the second term)
  auto kern = attn_kernel<DH, NW, MODE>;
  static std::atomic<unsigned> seen{0};
  if (first_use_on_device(seen))
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  hipLaunchKernelGGL(kern, dim3(a.n_tiles * a.n_heads), dim3(NW * 64), lds, s, a);
}

void launch_attention(hipStream_t s, const AttnArgs& a) {
  if (a.n_tiles == 0) return;
  const bool w8 = a.q_per_tile == 256, d64 = a.head_dim == 64;
#define ATTN_DISPATCH(M)                                                                       \
  do {                                                                                         \
    if (w8) { if (d64) launch_t<64, 8, M>(s, a); else launch_t<128, 8, M>(s, a); }             \
    else { if (d64) launch_t<64, 4, M>(s, a); else launch_t<128, 4, M>(s, a); }                \
  } while (0)
  if (a.mode == 3) {       // encoder attention: sequences are short, 128-query tiles only
    if (d64) launch_t<64, 4, 3>(s, a); else launch_t<128, 4, 3>(s, a);
  }
  else if (a.mode == 4) ATTN_DISPATCH(4);
  else if (a.mode == 2) ATTN_DISPATCH(2);
  else if (a.mode == 1) ATTN_DISPATCH(1);
  else ATTN_DISPATCH(0);
#undef ATTN_DISPATCH
}

}  // namespace dit
