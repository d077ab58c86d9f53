// Internal declarations shared by the host runtime and the kernel translation units.
// Not part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>

namespace dit {

typedef uint16_t bf16_t;  // storage type of bf16 tensors

// A kernel's dynamic-LDS limit is a per-device attribute: true the first time the calling thread's
// current device is seen for `mask` (one mask per kernel instantiation; devices 0..31).
inline bool first_use_on_device(std::atomic<unsigned>& mask) {
  int dev = 0;
  (void)hipGetDevice(&dev);
  const unsigned bit = 1u << (dev & 31);
  return (mask.fetch_or(bit) & bit) == 0;
}

// ---- GEMM ---------------------------------------------------------------------------
enum { OUT_BF16 = 0, OUT_F32 = 1, OUT_GELU_BF16 = 2, OUT_RESID_F32 = 3, OUT_QKNORM = 4 };

// OUT_QKNORM (only in the tile variants whose waves own 64 output columns): output columns [0, nq) are
// queries and [nq, nq+nk) keys: per head RMS norm (eps
// 1e-6) times gain, rotary code, queries times qscale, written as bf16 to qo / ko at row
// dst_row[m] (or m), column = column inside the q (k) range.  Columns from nq+nk on are written
// as OUT_BF16 to `out`.  nq and nk are multiples of 256, head_dim is 64 or 128.
struct QkNorm {
  int nq, nk, head_dim;
  const float* qgain; const float* kgain;   // [head_dim]
  const float2* rope;                       // [destination rows][head_dim/2] (cos, sin), or null
  const int* dst_row;                       // [M] or null
  bf16_t* qo; bf16_t* ko; int ldo;
  float qscale;
  int f16 = 0;                              // store q / k as fp16 instead of bf16
  // optional: the value columns (from nq+nk on) go out TRANSPOSED instead of to `out`:
  // vt[(n - nq - nk) * ldvt + vt_col[m]] = bf16(acc + bias); columns of vt that no row maps to are left alone
  bf16_t* vt = nullptr; int ldvt = 0;
  const int* vt_col = nullptr;              // [M]
};

struct GemmProblem {
  const bf16_t* A; int lda;     // [M][lda] activations
  const bf16_t* W; int ldw;     // [N_pad][ldw] weights, out-major
  const float* bias;            // [N] or null
  int M, N, K;
  int out_kind; void* out; int ldc;
  const float* gate; int gate_stride; const int* row_req;  // OUT_RESID_F32 only
  QkNorm qk;                                               // OUT_QKNORM only
  // 3x3 convolution as a product (conv_w > 0): A is a stack of channels-last bf16 images with a
  // one-pixel zero border each, [B][(H+2)*(conv_w+2)][conv_cin]; conv_img = H*conv_w pixels per
  // image; row m of the product is pixel (r / conv_w, r % conv_w) of image m / conv_img,
  // r = m % conv_img; column index k = tap*conv_cin + c with tap = 3*ky + kx; conv_cin % 64 == 0,
  // K = 9*conv_cin.  conv_kt = 3: a causal 3x3x3 convolution over a stack of frames: K = 27*conv_cin,
  // tap = (kf*3 + ky)*3 + kx, and frame tap kf of output frame b reads stack image b + kf, so A starts
  // with the two (zero) frames before the first.
  int conv_w = 0, conv_cin = 0, conv_img = 1, conv_kt = 1;
  // convolutions with OUT_F32 / OUT_RESID_F32 only, optional: per column n, the sum and the sum
  // of squares of the stored values over the rows of each (tile row, wave row) pair:
  // stats[(tile_row * 2 + wave_row)][N][2], rows of a pair = tile height / 2 (gemm_stats_rows)
  float* stats = nullptr;
  int tiles_m, tiles_n, tile_start;                        // filled by the launcher
};
struct GemmBatch {
  int n; int total_tiles; GemmProblem p[3];
  int splits = 1;                // split-K shares (chosen by the launcher)
  float* partial = nullptr;      // device scratch for split-K partial tiles, or null (no split-K)
  size_t partial_bytes = 0;
};

// Launches up to 3 independent problems in one grid.  Returns the tile shape used (BM*1000+BN).
int launch_gemm(hipStream_t s, GemmBatch& b, int force_tile = 0);
inline int gemm_stats_rows(int tile_code) { return (tile_code % 1000000) / 1000 / 2; }   // rows per stats chunk

// ---- attention ----------------------------------------------------------------------
// One block of q_per_tile queries of one segment.  parts == 0: against all keys of the segment.  parts > 0:
// share `part` of `parts` of the key tiles, kt0 .. kt0 + nkt - 1 (tiles of 64 keys); the shares of one block
// have the same `slot`, leave their unnormalised sums in AttnArgs::part and the last one to finish adds
// them in the order of `part` and writes the output rows.
struct AttnTile { int seg; int q0; int kt0; int nkt; int parts; int part; int slot; };
int attn_q_per_tile(int longest_segment, int head_dim);   // 128 or 256 queries per workgroup
struct AttnArgs {
  const bf16_t* q; int ldq;
  const bf16_t* k; int ldk;
  const bf16_t* vt; int ldvt;   // [H][dh][ldvt]
  bf16_t* o; int ldo;
  int n_heads, head_dim;
  const int* cu_q; const int* cu_k; const int* vt_off;   // device
  const AttnTile* tiles; int n_tiles;                    // device
  int q_per_tile;                                        // 128 (4 waves) or 256 (8 waves)
  // optional scatter of output rows: row j of segment s goes to o_row = map(...)
  const int* o_row_map;         // device [Nq] or null (identity)
  float scale_log2;             // log2(e)/sqrt(dh)
  int mode;                     // 0: q unscaled, running max; 1: q rows carry scale_log2, running max;
                                // 2: as 1 and |q.k| <= 60 for every pair: no running max at all;
                                // 3: as 0 plus bias[head][key - query + bias_L - 1] added to the scores
                                // 4: as 1 with q and k stored as fp16 and the values as two bf16 terms vt + vt_lo
  const float* bias = nullptr;  // mode 3: dev [n_heads][2*bias_L - 1]
  int bias_L = 0;               // mode 3: no segment is longer than this
  const bf16_t* vt_lo = nullptr; // mode 4: second term of the transposed values, same layout as vt
  // Key-split blocks (mode 2 only: without a running max the shares of a block simply add).
  int hpx = 0;                   // > 0: n_heads == 8 * hpx and workgroups run tile-major inside each group of hpx heads
                                 // (one group per XCD), so that the shares, last in the tile list, are the tail of every XCD
  int n_slots = 0;               // blocks that are split (AttnTile::slot < n_slots)
  float* part = nullptr;         // dev [n_heads][n_slots][parts][q_per_tile * (head_dim + 1)] floats
  unsigned* part_cnt = nullptr;  // dev [n_heads][n_slots], zero before the launch and zero again after it
};
void launch_attention(hipStream_t s, const AttnArgs& a);

// ---- row-wise / elementwise ---------------------------------------------------------
void launch_ln_modulate(hipStream_t s, const float* x, bf16_t* y, int M, int d,
                        const float* shift, const float* scale, int mod_stride,
                        const int* row_req, const float* gain, const float* beta,
                        bf16_t* y_lo = nullptr,    // optional second bf16 term (value - y)
                        int split = -1, const float* shift2 = nullptr, const float* scale2 = nullptr);
                        // rows >= split use shift2/scale2 (two streams in one launch)

// q/k per-head RMS norm (+ rotary) from a [M][ld] bf16 matrix holding q at column 0, k at
// column d; writes rows to qo/ko at row dst_row[m] (or m).  rope: [n_dst_rows][dh/2] (cos,sin)
// indexed by destination row, or null.
void launch_qknorm_rope(hipStream_t s, const bf16_t* qkv, int ld, int M, int H, int dh,
                        const float* qgain, const float* kgain, const float2* rope,
                        const int* dst_row, bf16_t* qo, bf16_t* ko, int ldo, int k_col_off,
                        int do_k, int split = -1, const float* qgain2 = nullptr,
                        const float* kgain2 = nullptr,    // rows >= split use the second gains
                        float qscale = 1.f);              // extra factor on the q output only

// V transpose: v rows [M][ld] at column v_col_off (+h*dh) -> vt[h][c][col], col = vt_col[m].
// Tiles of 64 destination columns; tile t covers columns 64t..64t+63 and takes source
// rows src_of_col[col] (-1 = write zero).
void launch_v_transpose(hipStream_t s, const bf16_t* v, int ld, int v_col_off, int H, int dh,
                        const int* src_of_col, int n_cols_pad, bf16_t* vt, int ldvt);

void launch_latent_update(hipStream_t s, float* x, const float* v, long long n, float a, float b);

// y[m][out_off_j + n] = sum_k f(x[m][k]) W_j[n][k] + b_j[n] for a device table of matrices sharing x (few rows
// M: one launch reads every matrix once); f = SiLU if silu_in.  x fp32 [M][ldx], W_j bf16 [N_j][ldw_j], y fp32
// [M][ldy].  Needs K % 8 == 0, ldx % 4 == 0, ldw_j % 8 == 0; returns false (nothing launched) otherwise.
struct SkinnyMat { const bf16_t* W; const float* bias; int N, ldw, out_off, pad; };
bool launch_skinny(hipStream_t s, const float* x, int ldx, const SkinnyMat* dev_mats, int n_mats, int max_n,
                   float* y, int ldy, int M, int K, int silu_in);

void launch_timestep_features(hipStream_t s, const float* sigma_dev, float* out, int M);
void launch_silu_split(hipStream_t s, const float* x, bf16_t* hi, bf16_t* lo, long long n, int silu = 1);   // hi + lo = SiLU(x) or x
// cross-attention keys (per-head RMS norm * gain, fp16) and transposed values (two bf16 terms) from
// the fp32 product kv[M][ld] = [keys | values]; vt_*: [H][dh][ldvt], column c takes row src_of_col[c]
void launch_cross_kv_finish(hipStream_t s, const float* kv, int ld, int M, int H, int dh, const float* kgain,
                            bf16_t* k16, int ldk, const int* src_of_col, int n_cols_pad, bf16_t* vt_hi,
                            bf16_t* vt_lo, int ldvt);

// patchify: latents fp32 packed -> bf16 [n_img][ldp] (columns >= pdim zero)
struct TokInfo { int req; int f, i, j; };  // per image token: request and grid position
void launch_patchify(hipStream_t s, const float* lat, const long long* lat_off_dev,
                     const int4* req_dims_dev /* (F,H,W,unused) per req */,
                     const TokInfo* tok, int n_img, int C, int pt, int ph, int pw,
                     bf16_t* out, bf16_t* out_lo, int ldp);   // out + out_lo = latent to ~16 bits
// x[m][c] += PE(i,j)[c] for family J
void launch_add_pe(hipStream_t s, float* x, const TokInfo* tok, int n_img, int d);
// unpatchify + update: for every latent element: v = y[token][feat]; x = a x + b v
void launch_unpatchify_update(hipStream_t s, float* lat, float* v_out, const float* y, int ldy,
                              const long long* lat_off_dev, const int4* req_dims_dev,
                              const int* img_off_dev, const float* a_dev, const float* b_dev,
                              int n_req, long long total, int C, int pt, int ph, int pw);
// rope table: out[row][j] = (cos, sin) of pos-dependent angle; rows with tok_of_row < 0 get (1,0)
void launch_rope_table(hipStream_t s, const TokInfo* tok, const int* tok_of_row, int n_rows,
                       int dh, int ax0, int ax1, int ax2, float theta, float2* out);
// out[m][:] = table[(m % 1)...] helpers for family W: e[r][6d] = base[r][6d] + table[6d]
void launch_add_rows(hipStream_t s, const float* base, int ld_base, const float* table,
                     float* out, int ld_out, int M, int N);
// gather rows: dst[dst_row[m]] = src[m] (fp32, d columns); either map may be null
void launch_copy_rows_f32(hipStream_t s, const float* src, const int* src_row, float* dst,
                          const int* dst_row, int M, int d);

// ---- Encode stage (text encoder) --------------------------------------------------------
void launch_embed_gather(hipStream_t s, const int* tokens, const float* table, float* x, int M, int d, int vocab);
// y = x / sqrt(mean(x^2) + 1e-6) * gain; y (bf16) and y32 (fp32) are each optional; d % 256 == 0
void launch_rmsnorm(hipStream_t s, const float* x, const float* gain, bf16_t* y, float* y32, int M, int d);
void launch_geglu(hipStream_t s, const bf16_t* a, const bf16_t* b, bf16_t* out, long long n);   // n % 8 == 0
// bias[h][delta + L - 1] = table[bucket(delta)][h] for delta in (-L, L); table fp32 [32][H]
void launch_rel_bias_table(hipStream_t s, const float* table, float* bias, int H, int L);

// ---- Decode stage (convolutional decoder), channels-last activations ----------------------
// latent fp32 [C][H][W] -> bf16 bordered image [(H+2)(W+2)][Cpad] (interior only; caller zero-fills)
// frames = 0: z is [B][C][H][W]; frames = B: z is one video [C][B][H][W]
void launch_latent_to_image(hipStream_t s, const float* z, bf16_t* out, int C, int H, int W, int Cpad, int B = 1, int frames = 0);
void launch_zero_border(hipStream_t s, bf16_t* img, int H, int W, int C, int B = 1);   // C % 8 == 0
// GroupNorm (eps 1e-6, affine) of the fp32 stream x [H*W][C], optional SiLU, bf16 output with
// (pad=1) or without a one-pixel border.  C in {64,128,256,512,1024}; partial: scratch of
// group_norm_partial_bytes; stats: scratch of GN_STATS_BYTES (groups <= 32).  ready_chunks > 0: partial already holds
// [ready_chunks][C][2] channel sums of x (GemmProblem::stats) and the statistics pass is skipped.
size_t group_norm_partial_bytes(long long pixels, int C);
constexpr int GN_MAX_BATCH = 128;
constexpr size_t GN_STATS_HEAD = (size_t)GN_MAX_BATCH * 32 * 8;                       // [B][groups] float2
constexpr size_t GN_STATS_BYTES = GN_STATS_HEAD + (size_t)GN_MAX_BATCH * 32 * 16 * 16;   // + [B][groups][shares] double2
void launch_group_norm(hipStream_t s, const float* x, const float* gamma, const float* beta, bf16_t* out,
                       float* partial, float2* stats, int H, int W, int C, int groups, int silu, int pad,
                       int ready_chunks = 0, int B = 1);   // B same-size images back to back, statistics per image
// nearest 2x upsampling of x [H*W][C] fp32 into a bf16 bordered image of size 2H x 2W
// B output images; frame_up: output image g shows input image (g + 1) / 2 (frame-rate doubling), else image g
void launch_upsample_pad(hipStream_t s, const float* x, bf16_t* out, int H, int W, int C, int B = 1, int frame_up = 0);
void launch_cast_bf16(hipStream_t s, const float* x, bf16_t* out, long long n);     // n % 4 == 0
// out[r][j] = softmax_j(sc[r][j] * scale) as bf16, j < n; columns n..ldo-1 are set to zero
void launch_softmax_rows(hipStream_t s, const float* sc, int lds_, bf16_t* out, int ldo, int rows, int n, float scale_log2);
// 3x3 convolution of a bordered bf16 image to OC <= 4 fp32 channels without the matrix cores;
// false (nothing launched) if the shape is outside its limits (C in {64,128,256,512}, OC <= 4).
// accumulate: out += instead of out = (one launch per frame tap of a 3x3x3 convolution).
bool launch_conv3_small(hipStream_t s, const bf16_t* img, const bf16_t* w, int ldw, const float* bias, float* out,
                        int H, int W, int C, int OC, int B = 1, int accumulate = 0);
void launch_compact_rows(hipStream_t s, const float* src, int lds_, float* dst, long long P, int C);

// weights
void launch_init_matrix(hipStream_t s, bf16_t* w, int rows_out, int cols_in, int ldw,
                        uint64_t key, float std);   // element (o,i) from logical index i*rows_out+o
void launch_init_table_f32(hipStream_t s, float* w, long long n, uint64_t key, float std);
void launch_fill_f32(hipStream_t s, float* p, long long n, float v);
void launch_fill_u16(hipStream_t s, bf16_t* p, long long n, uint16_t v);

}  // namespace dit
