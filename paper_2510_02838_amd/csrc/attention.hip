// Flash-style attention over packed variable-length segments on the gfx950 matrix cores.
//
//   O[q] = sum_k softmax_k(Q[q].K[k] / sqrt(dh)) V[k]      per segment and head, no mask
//
// never materialising the score matrix: keys are walked in tiles of 64 with the running
// max / running sum recurrence in fp32.
//
// Work split.  A workgroup of 4 waves owns 128 consecutive queries of one (segment, head);
// each wave owns 32 of them.  K tiles [64 keys][dh] and transposed-V tiles [dh][64 keys]
// stream through a double-buffered LDS ring via direct global->LDS loads.
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
#include <cstdlib>

namespace dit {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

static constexpr int KT = 64;     // keys per tile
static constexpr int QB = 128;    // queries per workgroup

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

template <int DH, int OCC>
__global__ __launch_bounds__(256, OCC) void attn_kernel(const AttnArgs a) {
  constexpr int KROW = DH * 2;                 // bytes per K-tile row
  constexpr int KCPR = DH / 8;                 // 16-byte chunks per K-tile row
  constexpr int KBYTES = KT * KROW;            // K tile
  constexpr int VBYTES = DH * 128;             // V^T tile: DH rows of 64 keys
  constexpr int STAGE = KBYTES + VBYTES;
  constexpr int LK = KT * KCPR / 256;          // chunks per thread, K tile
  constexpr int LV = DH * 8 / 256;             // chunks per thread, V^T tile
  constexpr int ND = DH / 32;                  // output d-tiles
  constexpr int NKK = DH / 16;                 // k-steps of the score product
  extern __shared__ __attribute__((aligned(128))) unsigned char smem[];

  // ---- which (tile, head) ------------------------------------------------------------
  int bid = blockIdx.x;
  {
    int nb = gridDim.x, x = bid & 7, idx = bid >> 3, q = nb >> 3, rem = nb & 7;
    bid = x * q + (x < rem ? x : rem) + idx;
  }
  const int head = bid / a.n_tiles;
  const AttnTile tile = a.tiles[bid - head * a.n_tiles];
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
    int q = i * 256 + tid, r = q / KCPR, pc = q % KCPR;
    int c = (DH == 64) ? (pc ^ ((r >> 1) & 7)) : (pc ^ (r & 15));
    krow[i] = r;
    gk[i] = head * DH + c * 8;
  }
#pragma unroll
  for (int i = 0; i < LV; ++i) {
    int q = i * 256 + tid, r = q >> 3, pc = q & 7, c = pc ^ ((r >> 1) & 7);
    gv[i] = (uint32_t)(head * DH + r) * (uint32_t)a.ldvt + vcol0 + c * 8;
  }
  const int n_kt = (klen + KT - 1) / KT;
  auto issue = [&](int kt, unsigned char* dst) {
#pragma unroll
    for (int i = 0; i < LK; ++i) {
      int key = kt * KT + krow[i];
      if (key >= klen) key = klen - 1;      // clamped rows are masked below
      const bf16_t* src = a.k + (size_t)(kbeg + key) * a.ldk + gk[i];
      __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)(dst + (i * 256 + wave * 64) * 16), 16, 0, 0);
    }
    const bf16_t* vsrc = a.vt + kt * KT;
#pragma unroll
    for (int i = 0; i < LV; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(vsrc + gv[i]), (lptr_t)(dst + KBYTES + (i * 256 + wave * 64) * 16), 16, 0, 0);
  };

  // ---- LDS read offsets ------------------------------------------------------------------
  // K operand row rho = l32 reads key kappa(rho): bits 2 and 3 swapped.
  const int kap = (l32 & ~12) | ((l32 & 8) >> 1) | ((l32 & 4) << 1);
  int koff[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) koff[t] = (kap + 32 * t) * KROW;
  const int kkey0 = (DH == 64) ? ((kap >> 1) & 7) : (kap & 15);   // (+32t does not change it)
  const int vkey = (l32 >> 1) & 7;                                 // (+32*dt does not change it)

  f32x16 o[ND];
#pragma unroll
  for (int d = 0; d < ND; ++d)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[d][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c2 = a.scale_log2;

  issue(0, smem);
  for (int kt = 0; kt < n_kt; ++kt) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (kt + 1 < n_kt) issue(kt + 1, smem + ((kt + 1) & 1) * STAGE);
    const unsigned char* sK = smem + (kt & 1) * STAGE;
    const unsigned char* sV = sK + KBYTES;

    // ---- S^T = K Q^T --------------------------------------------------------------------
    f32x16 st[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) st[t][e] = 0.f;
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
      const int c = kk * 2 + half;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        bf16x8 kf = *(const bf16x8*)(sK + koff[t] + ((c ^ kkey0) << 4));
        st[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], st[t], 0, 0, 0);
      }
    }
    // register e of tile t holds key  kt*64 + 32t + 16*(e/8) + 8*half + e%8
    if ((kt + 1) * KT > klen) {
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          int key = kt * KT + 32 * t + 16 * (e >> 3) + 8 * half + (e & 7);
          if (key >= klen) st[t][e] = -INFINITY;
        }
    }
    // ---- online softmax -------------------------------------------------------------------
    // The running max is only raised when some row's tile max exceeds it by more than 2^8 in
    // the exponent (softmax is shift-invariant, so a stale max is exact as long as nothing
    // overflows: probabilities stay below 2^8); this skips the rescale of O on most tiles.
    float mx = fmaxf(st[0][0], st[1][0]);
#pragma unroll
    for (int e = 1; e < 16; ++e) mx = fmaxf(mx, fmaxf(st[0][e], st[1][e]));
    mx = xhalf_max(mx);
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
    const float mc = m_run * c2;
    uint32_t pk[2][8];
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int e = 0; e < 16; e += 2) {
        const float p0 = __builtin_amdgcn_exp2f(st[t][e] * c2 - mc);
        const float p1 = __builtin_amdgcn_exp2f(st[t][e + 1] * c2 - mc);
        const uint32_t w = pack2bf(p0, p1);
        pk[t][e >> 1] = w;
        l_run = __builtin_amdgcn_fdot2_f32_bf16(*(const bf16x2*)&w, ones, l_run, false);  // sum of the rounded values
      }
    // ---- O^T += V^T P^T -------------------------------------------------------------------
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      union { uint32_t u[4]; bf16x8 v; } pf;
#pragma unroll
      for (int j = 0; j < 4; ++j) pf.u[j] = pk[s >> 1][(s & 1) * 4 + j];
      const int c = 2 * s + half;
#pragma unroll
      for (int d = 0; d < ND; ++d) {
        bf16x8 vf = *(const bf16x8*)(sV + (d * 32 + l32) * 128 + ((c ^ vkey) << 4));
        o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf.v, o[d], 0, 0, 0);
      }
    }
  }

  // ---- normalise and store -------------------------------------------------------------------
  const float l_tot = xhalf_sum(l_run);
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

template <int DH, int OCC>
static void launch_t(hipStream_t s, const AttnArgs& a) {
  constexpr int lds = 2 * (KT * DH * 2 + DH * 128);
  auto kern = attn_kernel<DH, OCC>;
  static bool done = false;
  if (!done) {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    done = true;
  }
  hipLaunchKernelGGL(kern, dim3(a.n_tiles * a.n_heads), dim3(256), lds, s, a);
}

void launch_attention(hipStream_t s, const AttnArgs& a) {
  if (a.n_tiles == 0) return;
  const char* e = getenv("DIT_ATTN_OCC");
  const int occ = e ? atoi(e) : 2;
  if (a.head_dim == 64) { if (occ == 3) launch_t<64, 3>(s, a); else if (occ == 4) launch_t<64, 4>(s, a); else launch_t<64, 2>(s, a); }
  else launch_t<128, 2>(s, a);
}

}  // namespace dit
