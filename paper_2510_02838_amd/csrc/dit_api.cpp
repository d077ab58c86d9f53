// Host runtime and C ABI of the Diffuse-stage library: tensor table, workspace carving,
// the per-step launch sequence for the three block families, taps and event profiling.
// Every arithmetic step of the denoising path runs in the HIP kernels; this file only
// validates, lays out memory and enqueues launches.
#include "../../include/dit.h"
#include "dit_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <cstdlib>
#include <map>
#include <string>
#include <unordered_map>
#include <vector>

using namespace dit;

namespace dit {
// Queries per attention workgroup.  256 (8 waves) halves the K/V traffic into LDS per query and
// measured 5% faster at 32760 tokens with head_dim 128; 128 (4 waves) gives twice as many
// workgroups, which wins on short sequences.  DIT_ATTN_QB=128|256 overrides.
int attn_q_per_tile(int longest_segment, int head_dim) {
  static const int forced = [] { const char* e = getenv("DIT_ATTN_QB"); return e ? atoi(e) : 0; }();
  if (forced == 128 || forced == 256) return forced;
  return (head_dim == 128 && longest_segment >= 16384) ? 256 : 128;
}
}  // namespace dit

namespace {

constexpr int T_FREQ = 256;   // width of the sinusoidal timestep feature
inline size_t rup(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct TensorRec {
  std::string name;
  int rows_in, cols_out, kind;   // kind: 0 matrix, 1 bias, 2 gain, 3 table
  size_t off;                    // byte offset in the arena
  int ld, rows_pad;              // matrices: leading dimension (elements) and padded out-rows
};

struct Tap { void* dst; size_t cap; int rows, cols, elem; };

// Everything derived from the list of requests of one call.
struct Plan {
  int n_req = 0;
  std::vector<dit_req> reqs;
  bool has_txt_stream = false;          // J, F: text tokens carry a residual stream
  int Nt = 0, Ni = 0, Ns = 0, Nj = 0;   // text rows, image rows, stream rows, joint rows
  int Nv_pad = 0, Nvx_pad = 0;          // V^T columns (self, cross)
  int qb = 128;                         // queries per attention workgroup
  long long lat_total = 0;
  std::vector<int> cu_txt, cu_img, cu_joint, vt_off, vtx_off;
  std::vector<long long> lat_off;
  std::vector<AttnTile> tiles, xtiles;
  std::vector<AttnTile> tiles_split;    // `tiles` with the blocks of the last, partly filled round split along the keys (or empty)
  int split_slots = 0, split_parts = 1;
  double attn_flop = 0, xattn_flop = 0;  // per head-dim unit: 4 * sum(nq*nk) * d
  // device copies (offsets into the workspace meta region)
  size_t o_cu_txt, o_cu_img, o_cu_joint, o_vt_off, o_vtx_off, o_lat_off, o_req_dims, o_tok, o_row_req_s,
      o_row_req_j, o_s2j, o_j2s, o_src_of_col, o_src_of_col_j, o_src_of_col_x, o_tok_of_row, o_tiles, o_xtiles,
      o_txt_rows, o_vtcol_s, o_vtcol_j, o_tiles_split, o_split_cnt, o_skinny;
  size_t meta_bytes = 0;
  std::vector<unsigned char> meta;       // host image of the meta region
};

struct WsLayout {
  size_t meta, sig, coef_a, coef_b, feat, th1, vec, mhi, mlo, mod, modblk, x, xj, xt0, h, qkv, q, k, vt, xk, vtx, vtlo, o, act, cproj,
      patch, yfin, rope, partial, attn_part, total;
  int MC = 0;        // modulation columns per conditioning row
  int R = 0;         // conditioning rows = steps * n_req
  int ldp = 0, ldy = 0;
};

}  // namespace

struct dit_ctx {
  dit_config cfg;
  int device = 0;
  hipStream_t stream = nullptr;
  std::vector<TensorRec> tensors;
  std::unordered_map<std::string, int> index;
  size_t weight_bytes = 0;
  unsigned char* weights = nullptr;
  unsigned char* ws = nullptr;
  size_t ws_bytes = 0;
  mutable std::string err;
  std::map<std::string, Tap> taps;
  // profiling
  bool prof = false;
  std::vector<hipEvent_t> ev_pool;
  struct Rec { int klass; };
  std::vector<Rec> ev_recs;
  double prof_flop[DIT_PROF_NCLASS] = {0}, prof_bytes[DIT_PROF_NCLASS] = {0};
  // cached plan (host side only) and a ring of host images for the per-call parameter upload
  Plan plan;
  bool plan_valid = false;
  struct Slot { std::vector<unsigned char> buf; hipEvent_t ev = nullptr; bool used = false; };
  Slot slots[4];
  int next_slot = 0;
  int pdim = 0;
  float* gemm_partial = nullptr;   // split-K scratch inside the workspace of the running call
  bool launch_refused = false;     // a product of the running call was outside the GEMM's limits
  int n_skinny = 0;                // entries of the conditioning-matrix table of the running call
  // largest |value| of every norm-gain vector (host copy, refreshed lazily after the weights change)
  std::unordered_map<std::string, float> gain_absmax;
  bool gain_stats_valid = false;
};

namespace {

dit_status fail(const dit_ctx* c, dit_status st, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c) c->err = buf;
  return st;
}

#define HIPCHK(c, call)                                                                             \
  do {                                                                                              \
    hipError_t e_ = (call);                                                                         \
    if (e_ != hipSuccess) return fail(c, DIT_EDEVICE, "%s: %s", #call, hipGetErrorString(e_));      \
  } while (0)

// ---------------------------------------------------------------------------------------
// tensor table
// ---------------------------------------------------------------------------------------
void add_tensor(dit_ctx* c, const std::string& name, int rows_in, int cols_out, int kind) {
  TensorRec t;
  t.name = name; t.rows_in = rows_in; t.cols_out = cols_out; t.kind = kind;
  t.off = c->weight_bytes;
  if (kind == 0) {
    t.ld = (int)rup(rows_in, 64);
    t.rows_pad = (int)rup(cols_out, 256);
    c->weight_bytes += rup((size_t)t.ld * t.rows_pad * 2, 256);
  } else {
    t.ld = cols_out; t.rows_pad = rows_in;
    c->weight_bytes += rup((size_t)rows_in * cols_out * 4, 256);
  }
  c->index[name] = (int)c->tensors.size();
  c->tensors.push_back(t);
}
void add_linear(dit_ctx* c, const std::string& p, int i, int o) {
  add_tensor(c, p + ".w", i, o, 0);
  add_tensor(c, p + ".b", 1, o, 1);
}
void add_stream_block(dit_ctx* c, const std::string& p) {
  const dit_config& g = c->cfg;
  add_linear(c, p + ".mod", g.hidden, 6 * g.hidden);
  add_linear(c, p + ".qkv", g.hidden, 3 * g.hidden);
  add_tensor(c, p + ".qnorm.g", 1, g.head_dim, 2);
  add_tensor(c, p + ".knorm.g", 1, g.head_dim, 2);
  add_linear(c, p + ".proj", g.hidden, g.hidden);
  add_linear(c, p + ".mlp1", g.hidden, g.mlp_hidden);
  add_linear(c, p + ".mlp2", g.mlp_hidden, g.hidden);
}
void build_table(dit_ctx* c) {
  const dit_config& g = c->cfg;
  const int d = g.hidden, dff = g.mlp_hidden;
  add_linear(c, "t_embed.1", T_FREQ, d);
  add_linear(c, "t_embed.2", d, d);
  add_linear(c, "x_embed", c->pdim, d);
  add_linear(c, "c_embed", g.cond_dim, d);
  char b[64];
  if (g.family == DIT_FAMILY_J || g.family == DIT_FAMILY_F) {
    const char* pre = g.family == DIT_FAMILY_J ? "blk" : "dbl";
    for (int l = 0; l < g.n_blocks; ++l)
      for (const char* s : {"txt", "img"}) {
        snprintf(b, sizeof b, "%s%d.%s", pre, l, s);
        add_stream_block(c, b);
      }
    for (int l = 0; l < g.n_single; ++l) {
      snprintf(b, sizeof b, "sgl%d", l);
      std::string p = b;
      add_linear(c, p + ".mod", d, 3 * d);
      add_linear(c, p + ".lin1", d, 3 * d + dff);
      add_tensor(c, p + ".qnorm.g", 1, g.head_dim, 2);
      add_tensor(c, p + ".knorm.g", 1, g.head_dim, 2);
      add_linear(c, p + ".lin2", d + dff, d);
    }
  } else {
    add_linear(c, "t_proj", d, 6 * d);
    for (int l = 0; l < g.n_blocks; ++l) {
      snprintf(b, sizeof b, "blk%d", l);
      std::string p = b;
      add_tensor(c, p + ".mod_table", 6, d, 3);
      add_linear(c, p + ".qkv", d, 3 * d);
      add_tensor(c, p + ".qnorm.g", 1, g.head_dim, 2);
      add_tensor(c, p + ".knorm.g", 1, g.head_dim, 2);
      add_linear(c, p + ".proj", d, d);
      add_tensor(c, p + ".xnorm.g", 1, d, 2);
      add_tensor(c, p + ".xnorm.b", 1, d, 1);
      add_linear(c, p + ".xq", d, d);
      add_linear(c, p + ".xkv", d, 2 * d);
      add_tensor(c, p + ".xqnorm.g", 1, g.head_dim, 2);
      add_tensor(c, p + ".xknorm.g", 1, g.head_dim, 2);
      add_linear(c, p + ".xproj", d, d);
      add_linear(c, p + ".mlp1", d, dff);
      add_linear(c, p + ".mlp2", dff, d);
    }
  }
  add_linear(c, "final.mod", d, 2 * d);
  add_linear(c, "final", d, c->pdim);
}

const TensorRec* find(const dit_ctx* c, const std::string& n) {
  auto it = c->index.find(n);
  return it == c->index.end() ? nullptr : &c->tensors[it->second];
}
const bf16_t* Wm(const dit_ctx* c, const std::string& n) { return (const bf16_t*)(c->weights + find(c, n)->off); }
const float* Wv(const dit_ctx* c, const std::string& n) { return (const float*)(c->weights + find(c, n)->off); }
int Wld(const dit_ctx* c, const std::string& n) { return find(c, n)->ld; }

// ---------------------------------------------------------------------------------------
// plan
// ---------------------------------------------------------------------------------------
dit_status validate_reqs(const dit_ctx* c, int n_req, const dit_req* reqs) {
  const dit_config& g = c->cfg;
  if (n_req <= 0 || !reqs) return fail(c, DIT_EINVAL, "n_req must be positive and reqs non-null");
  if (n_req > 4096) return fail(c, DIT_ESHAPE, "at most 4096 requests per call");
  long long tok = 0;
  for (int r = 0; r < n_req; ++r) {
    const dit_req& q = reqs[r];
    if (q.frames <= 0 || q.height <= 0 || q.width <= 0 || q.n_cond <= 0)
      return fail(c, DIT_ESHAPE, "request %d: empty latent or condition", r);
    if (q.frames % g.patch_t || q.height % g.patch_h || q.width % g.patch_w)
      return fail(c, DIT_ESHAPE, "request %d: latent extent not divisible by the patch", r);
    if (g.family == DIT_FAMILY_J && q.frames != 1)
      return fail(c, DIT_ESHAPE, "request %d: family J takes single-frame latents", r);
    tok += (long long)(q.frames / g.patch_t) * (q.height / g.patch_h) * (q.width / g.patch_w) + q.n_cond;
    if (tok > (1 << 20)) return fail(c, DIT_ESHAPE, "more than 2^20 tokens in one call");
  }
  // The kernels index activation matrices with 32-bit element offsets (row * row stride):
  // the widest matrix of the step must stay below 2^31 elements.
  const long long widest = std::max<long long>(3LL * g.hidden, (long long)g.hidden + g.mlp_hidden);
  if (tok * widest >= (1LL << 31))
    return fail(c, DIT_ESHAPE, "%lld tokens x %lld columns exceeds the 2^31-element activation limit", tok, widest);
  return DIT_OK;
}

template <class T>
size_t put(std::vector<unsigned char>& m, const std::vector<T>& v) {
  size_t off = rup(m.size(), 256);
  m.resize(off + std::max<size_t>(v.size() * sizeof(T), 4));
  if (!v.empty()) memcpy(m.data() + off, v.data(), v.size() * sizeof(T));
  return off;
}

// Key-split of the attention blocks in the last, partly filled round.  The chip's 8 XCDs take the workgroups
// of a launch in turn, each running its share in rounds of (32 CUs x workgroups per CU: 3 of 128 queries at
// head size 64, 2 at head size 128, 1 of 256 queries); when every block costs the same (requests of one
// shape) a launch of 1.1 rounds takes as long as one of 2.  The blocks of the partial round are cut into 2-4
// shares of their key tiles, so that this round is made of shorter workgroups that fill all CUs: 102 blocks
// per XCD on 96 slots become 96 whole blocks and 6 x 4 shares, 1 + 1/4 rounds.
// Needs a head count that is a multiple of 8 (each XCD owns whole heads: all shares of a block meet in one L2).
void plan_attention_split(Plan& P, const dit_config& g) {
  P.tiles_split.clear(); P.split_slots = 0; P.split_parts = 1;
  static const bool off = [] { const char* e = getenv("DIT_ATTN_SPLIT"); return e && atoi(e) == 0; }();
  if (off || P.tiles.empty() || g.n_heads % 8 != 0) return;
  const int klen = P.cu_joint[P.tiles[0].seg + 1] - P.cu_joint[P.tiles[0].seg];
  for (const AttnTile& t : P.tiles)
    if (P.cu_joint[t.seg + 1] - P.cu_joint[t.seg] != klen) return;       // mixed lengths: longest-first order handles the tail
  const int hpx = g.n_heads / 8, n_kt = (klen + 63) / 64;
  const int slots = 32 * (P.qb == 128 ? (g.head_dim == 64 ? 3 : 2) : 1);   // workgroups one XCD holds at a time
  const int per_xcd = (int)P.tiles.size() * hpx;
  const int rem = per_xcd % slots;
  if (per_xcd <= slots || rem == 0) return;
  const int t_split = std::min((int)P.tiles.size(), (rem + hpx - 1) / hpx);     // blocks per head that make up the partial round
  const int freed = (slots - (per_xcd - t_split * hpx) % slots) % slots;        // slots of the last full round the shares can use
  int best_parts = 1; double best = 1.0;
  for (int parts = 2; parts <= 4; ++parts) {
    if (n_kt < 8 * parts) break;
    const int items = t_split * hpx * parts - freed;
    const double cost = (double)((items + slots - 1) / slots) / parts + 0.04;   // rounds of the split part (+ writing and adding the shares)
    if (cost < best - 1e-9) { best = cost; best_parts = parts; }
  }
  if (best_parts == 1 || best > 0.75) return;      // (measured: 0.71 pays, -7 % attention time at 4250 tokens; 0.79 does not)
  const int n_whole = (int)P.tiles.size() - t_split;
  for (int i = 0; i < n_whole; ++i) P.tiles_split.push_back(P.tiles[i]);
  for (int i = 0; i < t_split; ++i)
    for (int pt = 0; pt < best_parts; ++pt) {
      AttnTile t = P.tiles[n_whole + i];
      t.kt0 = pt * n_kt / best_parts;
      t.nkt = (pt + 1) * n_kt / best_parts - t.kt0;
      t.parts = best_parts; t.part = pt; t.slot = i;
      P.tiles_split.push_back(t);
    }
  P.split_slots = t_split; P.split_parts = best_parts;
}

void build_plan(const dit_ctx* c, int n_req, const dit_req* reqs, Plan& P) {
  const dit_config& g = c->cfg;
  P = Plan();
  P.n_req = n_req;
  P.reqs.assign(reqs, reqs + n_req);
  P.has_txt_stream = g.family != DIT_FAMILY_W;
  P.cu_txt.assign(1, 0); P.cu_img.assign(1, 0); P.cu_joint.assign(1, 0); P.lat_off.assign(1, 0);
  std::vector<int4> req_dims;
  std::vector<TokInfo> tok;
  int vcol = 0, vxcol = 0;
  for (int r = 0; r < n_req; ++r) {
    const dit_req& q = reqs[r];
    const int gf = q.frames / g.patch_t, gh = q.height / g.patch_h, gw = q.width / g.patch_w;
    const int ni = gf * gh * gw, nt = q.n_cond;
    const int nj = ni + (P.has_txt_stream ? nt : 0);
    P.cu_txt.push_back(P.cu_txt.back() + nt);
    P.cu_img.push_back(P.cu_img.back() + ni);
    P.cu_joint.push_back(P.cu_joint.back() + nj);
    P.lat_off.push_back(P.lat_off.back() + (long long)g.latent_ch * q.frames * q.height * q.width);
    req_dims.push_back(make_int4(q.frames, q.height, q.width, 0));
    for (int f = 0; f < gf; ++f)
      for (int i = 0; i < gh; ++i)
        for (int j = 0; j < gw; ++j) tok.push_back(TokInfo{r, f, i, j});
    P.vt_off.push_back(vcol); vcol += (int)rup(nj, 64);
    P.vtx_off.push_back(vxcol); vxcol += (int)rup(nt, 64);
    P.attn_flop += 4.0 * nj * nj;
    P.xattn_flop += 4.0 * ni * nt;
  }
  P.Nt = P.cu_txt.back(); P.Ni = P.cu_img.back(); P.Nj = P.cu_joint.back();
  P.Ns = P.Ni + (P.has_txt_stream ? P.Nt : 0);
  P.Nv_pad = vcol; P.Nvx_pad = vxcol;
  P.lat_total = P.lat_off.back();
  const int soff_img = P.has_txt_stream ? P.Nt : 0;     // image rows follow text rows in the stream buffer

  std::vector<int> row_req_s(P.Ns), row_req_j(P.Nj), s2j(P.Ns), j2s(P.Nj), tok_of_row(P.Nj, -1);
  std::vector<int> src_of_col(P.Nv_pad, -1), src_of_col_j(P.Nv_pad, -1), src_of_col_x(P.Nvx_pad, -1);
  std::vector<int> txt_rows(std::max(P.Nt, 1));
  std::vector<int> vtcol_s(P.Ns), vtcol_j(P.Nj);      // V^T column of every stream row / joint row
  int longest = 0;
  for (int r = 0; r < n_req; ++r) longest = std::max(longest, P.cu_joint[r + 1] - P.cu_joint[r]);
  P.qb = attn_q_per_tile(longest, g.head_dim);
  for (int r = 0; r < n_req; ++r) {
    const int nt = P.cu_txt[r + 1] - P.cu_txt[r], ni = P.cu_img[r + 1] - P.cu_img[r];
    int j = P.cu_joint[r];
    if (P.has_txt_stream)
      for (int t = 0; t < nt; ++t, ++j) {
        const int s = P.cu_txt[r] + t;
        row_req_s[s] = r; s2j[s] = j; j2s[j] = s; row_req_j[j] = r;
      }
    for (int t = 0; t < ni; ++t, ++j) {
      const int s = soff_img + P.cu_img[r] + t;
      row_req_s[s] = r; s2j[s] = j; j2s[j] = s; row_req_j[j] = r;
      tok_of_row[j] = P.cu_img[r] + t;
    }
    const int nj = P.cu_joint[r + 1] - P.cu_joint[r];
    for (int t = 0; t < nj; ++t) {
      src_of_col[P.vt_off[r] + t] = j2s[P.cu_joint[r] + t];
      src_of_col_j[P.vt_off[r] + t] = P.cu_joint[r] + t;
      vtcol_j[P.cu_joint[r] + t] = P.vt_off[r] + t;
      vtcol_s[j2s[P.cu_joint[r] + t]] = P.vt_off[r] + t;
    }
    for (int t = 0; t < nt; ++t) src_of_col_x[P.vtx_off[r] + t] = P.cu_txt[r] + t;
    for (int q0 = 0; q0 < nj; q0 += P.qb) P.tiles.push_back(AttnTile{r, q0});
    for (int q0 = 0; q0 < ni; q0 += P.qb) P.xtiles.push_back(AttnTile{r, q0});
  }
  // longest key ranges first, so that the tail of the grid is made of short tiles
  std::stable_sort(P.tiles.begin(), P.tiles.end(), [&](const AttnTile& a, const AttnTile& b) {
    return P.cu_joint[a.seg + 1] - P.cu_joint[a.seg] > P.cu_joint[b.seg + 1] - P.cu_joint[b.seg];
  });
  plan_attention_split(P, g);
  std::vector<unsigned char>& m = P.meta;
  P.o_cu_txt = put(m, P.cu_txt); P.o_cu_img = put(m, P.cu_img); P.o_cu_joint = put(m, P.cu_joint);
  P.o_vt_off = put(m, P.vt_off); P.o_vtx_off = put(m, P.vtx_off); P.o_lat_off = put(m, P.lat_off);
  P.o_req_dims = put(m, req_dims); P.o_tok = put(m, tok);
  P.o_row_req_s = put(m, row_req_s); P.o_row_req_j = put(m, row_req_j);
  P.o_s2j = put(m, s2j); P.o_j2s = put(m, j2s);
  P.o_src_of_col = put(m, src_of_col); P.o_src_of_col_j = put(m, src_of_col_j);
  P.o_src_of_col_x = put(m, src_of_col_x); P.o_tok_of_row = put(m, tok_of_row);
  P.o_tiles = put(m, P.tiles); P.o_xtiles = put(m, P.xtiles);
  P.o_txt_rows = put(m, txt_rows);
  P.o_vtcol_s = put(m, vtcol_s); P.o_vtcol_j = put(m, vtcol_j);
  P.o_tiles_split = put(m, P.tiles_split);
  P.o_split_cnt = put(m, std::vector<unsigned>((size_t)g.n_heads * P.split_slots + 1, 0u));   // (uploaded as zeros with every call)
  // table of the conditioning matrices (timestep MLP, every modulation matrix): filled with arena addresses per call
  P.o_skinny = put(m, std::vector<SkinnyMat>((size_t)(2 * g.n_blocks + g.n_single + 4), SkinnyMat{nullptr, nullptr, 0, 0, 0, 0}));
  P.meta_bytes = rup(m.size(), 256);
  m.resize(P.meta_bytes);
}

int mod_cols(const dit_config& g) {
  const int d = g.hidden;
  if (g.family == DIT_FAMILY_J) return g.n_blocks * 12 * d + 2 * d;
  if (g.family == DIT_FAMILY_F) return g.n_blocks * 12 * d + g.n_single * 3 * d + 2 * d;
  return 6 * d + 2 * d;
}

// split-K scratch: at most 256 workgroups, each leaving one 128x128 fp32 tile
constexpr size_t GEMM_PARTIAL_BYTES = (size_t)256 * 128 * 128 * 4;

void layout_ws(const dit_ctx* c, const Plan& P, int max_steps, WsLayout& L) {
  const dit_config& g = c->cfg;
  const size_t d = g.hidden, dff = g.mlp_hidden;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += rup(bytes, 256); return at; };
  L.R = max_steps * P.n_req;
  L.MC = mod_cols(g);
  L.ldp = (int)rup(c->pdim, 64);
  L.ldy = (int)rup(c->pdim, 4);
  const size_t Ns = P.Ns, Nj = P.Nj, Nt = P.Nt, Ni = P.Ni;
  const size_t wide = (g.family == DIT_FAMILY_F && g.n_single > 0) ? d + dff : 0;
  L.meta = take(P.meta_bytes);
  L.sig = take((size_t)L.R * 4);
  L.coef_a = take((size_t)L.R * 4);
  L.coef_b = take((size_t)L.R * 4);
  L.feat = take((size_t)L.R * T_FREQ * 4);
  L.th1 = take((size_t)L.R * d * 4);
  L.vec = take((size_t)L.R * d * 4);
  L.mhi = take((size_t)L.R * d * 2);
  L.mlo = take((size_t)L.R * d * 2);
  L.mod = take((size_t)L.R * L.MC * 4);
  L.modblk = take((size_t)P.n_req * 6 * d * 4);
  L.x = take(Ns * d * 4);
  L.xj = take(g.family == DIT_FAMILY_F ? Nj * d * 4 : 0);
  L.xt0 = take(Nt * d * 4);                      // projected condition, fp32
  L.h = take(std::max(Ns, Nj) * d * 2);
  L.qkv = take(std::max(Ns, Nj) * 3 * d * 2);
  L.q = take(Nj * d * 2);
  L.k = take(std::max(Nj, Nt) * d * 2);
  L.vt = take(d * (size_t)P.Nv_pad * 2);         // self-attention values, transposed (pad columns stay zero for a whole call)
  // cross-attention keys (fp16) and transposed values (two bf16 terms) of EVERY block: they depend on the condition
  // only and are formed once per call, not once per step
  const size_t nbw = g.family == DIT_FAMILY_W ? (size_t)g.n_blocks : 0;
  L.xk = take(nbw * Nt * d * 2);
  L.vtx = take(nbw * d * (size_t)P.Nvx_pad * 2);     // first ...
  L.vtlo = take(nbw * d * (size_t)P.Nvx_pad * 2);    // ... and second term
  L.o = take(Ns * d * 2);
  L.act = take(std::max(std::max(Ns * dff, Nj * wide) * 2, Nt * 2 * d * 4));    // (family W: fp32 keys|values of the condition)
  L.cproj = take(g.family == DIT_FAMILY_W ? Nt * d * 2 * 2 : 0);               // projected condition as two bf16 terms
  L.patch = take(Ni * (size_t)L.ldp * 2 * 2);   // hi and lo terms
  L.yfin = take(Ni * (size_t)L.ldy * 4);
  L.rope = take((g.rope_axes[0] + g.rope_axes[1] + g.rope_axes[2]) > 0 ? Nj * (g.head_dim / 2) * 8 : 0);
  L.partial = take(GEMM_PARTIAL_BYTES);
  L.attn_part = take((size_t)g.n_heads * P.split_slots * P.split_parts * P.qb * (g.head_dim + 1) * 4);   // sums of key-split attention blocks
  L.total = o;
}

// ---------------------------------------------------------------------------------------
// launch helpers with profiling
// ---------------------------------------------------------------------------------------
struct Scope {
  dit_ctx* c; int klass; bool on; hipEvent_t end = nullptr;
  Scope(dit_ctx* c_, int k, double flop, double bytes) : c(c_), klass(k), on(c_->prof) {
    if (!on) return;
    c->prof_flop[k] += flop; c->prof_bytes[k] += bytes;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) { on = false; return; }
    c->ev_pool.push_back(e0); c->ev_pool.push_back(e1);
    c->ev_recs.push_back({k});
    end = e1;
    (void)hipEventRecord(e0, c->stream);
  }
  ~Scope() { if (on) (void)hipEventRecord(end, c->stream); }   // (scopes may nest)
};

GemmProblem mk(const bf16_t* A, int lda, const bf16_t* W, int ldw, const float* bias, int M, int N, int K,
               int kind, void* out, int ldc, const float* gate = nullptr, int gstride = 0,
               const int* row_req = nullptr) {
  GemmProblem p;
  p.A = A; p.lda = lda; p.W = W; p.ldw = ldw; p.bias = bias; p.M = M; p.N = N; p.K = K;
  p.out_kind = kind; p.out = out; p.ldc = ldc; p.gate = gate; p.gate_stride = gstride; p.row_req = row_req;
  p.tiles_m = p.tiles_n = p.tile_start = 0;
  p.qk = QkNorm{};
  return p;
}
// QKV-type product whose first nq (nk) output columns are normalised queries (keys) written to qo (ko)
GemmProblem with_qknorm(GemmProblem p, int nq, int nk, int head_dim, const float* qgain, const float* kgain,
                        const float2* rope, const int* dst_row, bf16_t* qo, bf16_t* ko, int ldo, float qscale) {
  p.out_kind = OUT_QKNORM;
  p.qk = QkNorm{nq, nk, head_dim, qgain, kgain, rope, dst_row, qo, ko, ldo, qscale};
  return p;
}
// ... and whose value columns go out transposed, row m to column vt_col[m] of vt[H*dh][ldvt]
GemmProblem with_vt(GemmProblem p, bf16_t* vt, int ldvt, const int* vt_col) {
  p.qk.vt = vt; p.qk.ldvt = ldvt; p.qk.vt_col = vt_col;
  return p;
}
void run_gemm(dit_ctx* c, std::initializer_list<GemmProblem> ps) {
  GemmBatch b;
  b.n = 0; b.total_tiles = 0;
  double flop = 0, bytes = 0;
  for (const GemmProblem& p : ps) {
    if (p.M <= 0 || p.N <= 0) continue;
    b.p[b.n++] = p;
    flop += 2.0 * p.M * p.N * p.K;
    bytes += 2.0 * ((double)p.M * p.K + (double)p.N * p.K) + (double)p.M * p.N * (p.out_kind == OUT_RESID_F32 ? 8 : p.out_kind == OUT_F32 ? 4 : 2);
  }
  if (!b.n) return;
  b.partial = c->gemm_partial; b.partial_bytes = c->gemm_partial ? GEMM_PARTIAL_BYTES : 0;
  Scope sc(c, DIT_PROF_GEMM, flop, bytes);
  if (launch_gemm(c->stream, b) < 0) c->launch_refused = true;     // shape outside the kernels' limits: reported by the call
}

dit_status do_tap(dit_ctx* c, const std::string& name, const void* src, int rows, int cols, int elem, int ld) {
  auto it = c->taps.find(name);
  if (it == c->taps.end()) return DIT_OK;
  Tap& t = it->second;
  const size_t need = (size_t)rows * cols * elem;
  if (need > t.cap) return fail(c, DIT_ENOMEM, "tap %s needs %zu bytes, buffer has %zu", name.c_str(), need, t.cap);
  t.rows = rows; t.cols = cols; t.elem = elem;
  HIPCHK(c, hipMemcpy2DAsync(t.dst, (size_t)cols * elem, src, (size_t)ld * elem, (size_t)cols * elem, rows,
                             hipMemcpyDeviceToDevice, c->stream));
  return DIT_OK;
}
#define TAP(name, src, rows, cols, elem, ld)                                         \
  do {                                                                               \
    if (!c->taps.empty()) {                                                          \
      dit_status st_ = do_tap(c, name, src, rows, cols, elem, ld);                   \
      if (st_ != DIT_OK) return st_;                                                 \
    }                                                                                \
  } while (0)

// ---------------------------------------------------------------------------------------
// the step
// ---------------------------------------------------------------------------------------
struct Run {
  dit_ctx* c; const Plan& P; const WsLayout& L; unsigned char* ws;
  template <class T> T* at(size_t off) const { return (T*)(ws + off); }
  const int* ip(size_t meta_off) const { return (const int*)(ws + L.meta + meta_off); }
};

// log2(e)/sqrt(dh): folded into the q rows by the q/k-norm kernel, so that scores are exponents
static inline float attn_qscale(int head_dim) { return 1.4426950408889634f / sqrtf((float)head_dim); }

static float gmax(const dit_ctx* c, const std::string& a, const std::string& b = std::string()) {
  auto one = [&](const std::string& n) {
    auto it = c->gain_absmax.find(n);
    return it == c->gain_absmax.end() ? INFINITY : it->second;   // unknown: no bound, keep the running max
  };
  float m = one(a);
  if (!b.empty()) m = std::max(m, one(b));
  return m;
}

void run_attention(dit_ctx* c, const Run& R, const bf16_t* q, int ldq, const bf16_t* k, int ldk, const bf16_t* vt,
                   int ldvt, bf16_t* o, int ldo, const int* cu_q, const int* cu_k, const int* vt_off,
                   const AttnTile* tiles, int n_tiles, const int* o_row_map, double flop_units,
                   float q_gain_max, float k_gain_max, const bf16_t* vt_lo = nullptr, bool split = false) {
  const dit_config& g = c->cfg;
  AttnArgs a;
  a.q = q; a.ldq = ldq; a.k = k; a.ldk = ldk; a.vt = vt; a.ldvt = ldvt; a.o = o; a.ldo = ldo;
  a.n_heads = g.n_heads; a.head_dim = g.head_dim; a.cu_q = cu_q; a.cu_k = cu_k; a.vt_off = vt_off;
  a.tiles = tiles; a.n_tiles = n_tiles; a.o_row_map = o_row_map; a.q_per_tile = R.P.qb;
  a.scale_log2 = attn_qscale(g.head_dim);
  // q and k are RMS-normalised per head, so |q'.k| <= (c sqrt(dh) max|g_q|) (sqrt(dh) max|g_k|) with c
  // the factor folded into q; 2 % on top for the bf16 rounding of both rows.  Below 60 the
  // attention kernel needs no running max.
  const float logit_bound = a.scale_log2 * (float)g.head_dim * q_gain_max * k_gain_max * 1.02f;
  a.mode = logit_bound <= 60.0f ? 2 : 1;
  if (vt_lo) { a.mode = 4; a.vt_lo = vt_lo; }    // fp16 q/k, two-term values, running max
  if (a.mode == 2 && split && R.P.split_slots > 0) {   // key-split blocks in the last round (they add without a running max)
    a.tiles = (const AttnTile*)(R.ws + R.L.meta + R.P.o_tiles_split); a.n_tiles = (int)R.P.tiles_split.size();
    a.hpx = g.n_heads / 8; a.n_slots = R.P.split_slots;
    a.part = R.at<float>(R.L.attn_part); a.part_cnt = (unsigned*)(R.ws + R.L.meta + R.P.o_split_cnt);
  }
  Scope sc(c, DIT_PROF_ATTN, flop_units * g.hidden, 0);
  launch_attention(c->stream, a);
}

// joint two-stream block (families J and F-double)
dit_status joint_block(dit_ctx* c, const Run& R, const std::string& p, const float* mod, int mod_off) {
  const dit_config& g = c->cfg;
  const Plan& P = R.P; const WsLayout& L = R.L;
  const int d = g.hidden, dff = g.mlp_hidden, Nt = P.Nt, Ni = P.Ni, Ns = P.Ns, MC = L.MC;
  float* x = R.at<float>(L.x);
  bf16_t* h = R.at<bf16_t>(L.h); bf16_t* qkv = R.at<bf16_t>(L.qkv);
  bf16_t* q = R.at<bf16_t>(L.q); bf16_t* k = R.at<bf16_t>(L.k); bf16_t* vt = R.at<bf16_t>(L.vt);
  bf16_t* o = R.at<bf16_t>(L.o); bf16_t* act = R.at<bf16_t>(L.act);
  const int* rreq = R.ip(P.o_row_req_s);
  const int* s2j = R.ip(P.o_s2j);
  const float2* rope = (g.rope_axes[0] + g.rope_axes[1] + g.rope_axes[2]) > 0 ? R.at<float2>(L.rope) : nullptr;
  const std::string pt = p + ".txt", pi = p + ".img";
  const float* mt = mod + mod_off;           // text stream: 6d
  const float* mi = mod + mod_off + 6 * d;   // image stream: 6d
  {
    Scope sc(c, DIT_PROF_LNMOD, 0, 6.0 * Ns * d);
    launch_ln_modulate(c->stream, x, h, Ns, d, mt, mt + d, MC, rreq, nullptr, nullptr, nullptr, Nt, mi, mi + d);
  }
  TAP(pt + ".ln1", h, Nt, d, 2, d); TAP(pi + ".ln1", h + (size_t)Nt * d, Ni, d, 2, d);
  // With no capture point registered the q/k norm, rotary code and softmax scale are the QKV
  // product's epilogue; with taps every intermediate is materialised by its own kernel.
  const bool fuse = c->taps.empty();
  const float qs = attn_qscale(g.head_dim);
  GemmProblem pq_t = mk(h, d, Wm(c, pt + ".qkv.w"), Wld(c, pt + ".qkv.w"), Wv(c, pt + ".qkv.b"), Nt, 3 * d, d, OUT_BF16, qkv, 3 * d);
  GemmProblem pq_i = mk(h + (size_t)Nt * d, d, Wm(c, pi + ".qkv.w"), Wld(c, pi + ".qkv.w"), Wv(c, pi + ".qkv.b"), Ni, 3 * d, d, OUT_BF16, qkv + (size_t)Nt * 3 * d, 3 * d);
  if (fuse) {
    const int* vtc = R.ip(P.o_vtcol_s);
    pq_t = with_vt(with_qknorm(pq_t, d, d, g.head_dim, Wv(c, pt + ".qnorm.g"), Wv(c, pt + ".knorm.g"), rope, s2j, q, k, d, qs), vt, P.Nv_pad, vtc);
    pq_i = with_vt(with_qknorm(pq_i, d, d, g.head_dim, Wv(c, pi + ".qnorm.g"), Wv(c, pi + ".knorm.g"), rope, s2j + Nt, q, k, d, qs), vt, P.Nv_pad, vtc + Nt);
  }
  run_gemm(c, {pq_t, pq_i});
  TAP(pt + ".qkv", qkv, Nt, 3 * d, 2, 3 * d); TAP(pi + ".qkv", qkv + (size_t)Nt * 3 * d, Ni, 3 * d, 2, 3 * d);
  if (!fuse) {
    Scope sc(c, DIT_PROF_QKNORM, 0, 12.0 * Ns * d);
    launch_qknorm_rope(c->stream, qkv, 3 * d, Ns, g.n_heads, g.head_dim, Wv(c, pt + ".qnorm.g"), Wv(c, pt + ".knorm.g"), rope, s2j, q, k, d, d, 1,
                       Nt, Wv(c, pi + ".qnorm.g"), Wv(c, pi + ".knorm.g"), qs);
    launch_v_transpose(c->stream, qkv, 3 * d, 2 * d, g.n_heads, g.head_dim, R.ip(P.o_src_of_col), P.Nv_pad, vt, P.Nv_pad);
  }
  TAP(p + ".q", q, P.Nj, d, 2, d); TAP(p + ".k", k, P.Nj, d, 2, d);
  run_attention(c, R, q, d, k, d, vt, P.Nv_pad, o, d, R.ip(P.o_cu_joint), R.ip(P.o_cu_joint), R.ip(P.o_vt_off),
                (const AttnTile*)(R.ws + L.meta + P.o_tiles), (int)P.tiles.size(), R.ip(P.o_j2s), P.attn_flop,
                gmax(c, pt + ".qnorm.g", pi + ".qnorm.g"), gmax(c, pt + ".knorm.g", pi + ".knorm.g"), nullptr, true);
  TAP(p + ".attn", o, Ns, d, 2, d);   // stream order: text rows, then image rows
  run_gemm(c, {mk(o, d, Wm(c, pt + ".proj.w"), Wld(c, pt + ".proj.w"), Wv(c, pt + ".proj.b"), Nt, d, d, OUT_RESID_F32, x, d, mt + 2 * d, MC, rreq),
               mk(o + (size_t)Nt * d, d, Wm(c, pi + ".proj.w"), Wld(c, pi + ".proj.w"), Wv(c, pi + ".proj.b"), Ni, d, d, OUT_RESID_F32, x + (size_t)Nt * d, d, mi + 2 * d, MC, rreq + Nt)});
  TAP(pt + ".x_attn", x, Nt, d, 4, d); TAP(pi + ".x_attn", x + (size_t)Nt * d, Ni, d, 4, d);
  {
    Scope sc(c, DIT_PROF_LNMOD, 0, 6.0 * Ns * d);
    launch_ln_modulate(c->stream, x, h, Ns, d, mt + 3 * d, mt + 4 * d, MC, rreq, nullptr, nullptr, nullptr, Nt, mi + 3 * d, mi + 4 * d);
  }
  run_gemm(c, {mk(h, d, Wm(c, pt + ".mlp1.w"), Wld(c, pt + ".mlp1.w"), Wv(c, pt + ".mlp1.b"), Nt, dff, d, OUT_GELU_BF16, act, dff),
               mk(h + (size_t)Nt * d, d, Wm(c, pi + ".mlp1.w"), Wld(c, pi + ".mlp1.w"), Wv(c, pi + ".mlp1.b"), Ni, dff, d, OUT_GELU_BF16, act + (size_t)Nt * dff, dff)});
  TAP(pt + ".mlp_act", act, Nt, dff, 2, dff); TAP(pi + ".mlp_act", act + (size_t)Nt * dff, Ni, dff, 2, dff);
  run_gemm(c, {mk(act, dff, Wm(c, pt + ".mlp2.w"), Wld(c, pt + ".mlp2.w"), Wv(c, pt + ".mlp2.b"), Nt, d, dff, OUT_RESID_F32, x, d, mt + 5 * d, MC, rreq),
               mk(act + (size_t)Nt * dff, dff, Wm(c, pi + ".mlp2.w"), Wld(c, pi + ".mlp2.w"), Wv(c, pi + ".mlp2.b"), Ni, d, dff, OUT_RESID_F32, x + (size_t)Nt * d, d, mi + 5 * d, MC, rreq + Nt)});
  TAP(pt + ".x_out", x, Nt, d, 4, d); TAP(pi + ".x_out", x + (size_t)Nt * d, Ni, d, 4, d);
  return DIT_OK;
}

// single-stream block of family F on the joint-ordered residual xj
dit_status single_block(dit_ctx* c, const Run& R, const std::string& p, const float* mod, int mod_off) {
  const dit_config& g = c->cfg;
  const Plan& P = R.P; const WsLayout& L = R.L;
  const int d = g.hidden, dff = g.mlp_hidden, Nj = P.Nj, MC = L.MC, wide = d + dff;
  float* xj = R.at<float>(L.xj);
  bf16_t* h = R.at<bf16_t>(L.h); bf16_t* qkv = R.at<bf16_t>(L.qkv);
  bf16_t* q = R.at<bf16_t>(L.q); bf16_t* k = R.at<bf16_t>(L.k); bf16_t* vt = R.at<bf16_t>(L.vt);
  bf16_t* cat = R.at<bf16_t>(L.act);
  const int* rreq = R.ip(P.o_row_req_j);
  const float2* rope = (g.rope_axes[0] + g.rope_axes[1] + g.rope_axes[2]) > 0 ? R.at<float2>(L.rope) : nullptr;
  const float* m = mod + mod_off;
  {
    Scope sc(c, DIT_PROF_LNMOD, 0, 6.0 * Nj * d);
    launch_ln_modulate(c->stream, xj, h, Nj, d, m, m + d, MC, rreq, nullptr, nullptr);
  }
  const bf16_t* w1 = Wm(c, p + ".lin1.w"); const int ld1 = Wld(c, p + ".lin1.w"); const float* b1 = Wv(c, p + ".lin1.b");
  const bool fuse = c->taps.empty();          // see joint_block
  const float qs = attn_qscale(g.head_dim);
  GemmProblem pq = mk(h, d, w1, ld1, b1, Nj, 3 * d, d, OUT_BF16, qkv, 3 * d);
  if (fuse) pq = with_vt(with_qknorm(pq, d, d, g.head_dim, Wv(c, p + ".qnorm.g"), Wv(c, p + ".knorm.g"), rope, nullptr, q, k, d, qs), vt, P.Nv_pad, R.ip(P.o_vtcol_j));
  run_gemm(c, {pq, mk(h, d, w1 + (size_t)3 * d * ld1, ld1, b1 + 3 * d, Nj, dff, d, OUT_GELU_BF16, cat + d, wide)});
  TAP(p + ".lin1", qkv, Nj, 3 * d, 2, 3 * d);
  if (!fuse) {
    Scope sc(c, DIT_PROF_QKNORM, 0, 12.0 * Nj * d);
    launch_qknorm_rope(c->stream, qkv, 3 * d, Nj, g.n_heads, g.head_dim, Wv(c, p + ".qnorm.g"), Wv(c, p + ".knorm.g"), rope, nullptr, q, k, d, d, 1,
                       -1, nullptr, nullptr, qs);
    launch_v_transpose(c->stream, qkv, 3 * d, 2 * d, g.n_heads, g.head_dim, R.ip(P.o_src_of_col_j), P.Nv_pad, vt, P.Nv_pad);
  }
  run_attention(c, R, q, d, k, d, vt, P.Nv_pad, cat, wide, R.ip(P.o_cu_joint), R.ip(P.o_cu_joint), R.ip(P.o_vt_off),
                (const AttnTile*)(R.ws + L.meta + P.o_tiles), (int)P.tiles.size(), nullptr, P.attn_flop,
                gmax(c, p + ".qnorm.g"), gmax(c, p + ".knorm.g"), nullptr, true);
  TAP(p + ".attn", cat, Nj, d, 2, wide);
  run_gemm(c, {mk(cat, wide, Wm(c, p + ".lin2.w"), Wld(c, p + ".lin2.w"), Wv(c, p + ".lin2.b"), Nj, d, wide, OUT_RESID_F32, xj, d, m + 2 * d, MC, rreq)});
  TAP(p + ".x_out", xj, Nj, d, 4, d);
  return DIT_OK;
}

// self-attention + cross-attention + MLP block of family W (image rows only in x)
// Keys and values of block `blk`'s cross-attention, from the two-term projected condition with fp32 results:
// keys RMS-normalised per head and stored as fp16, values transposed as two bf16 terms.  Step-invariant.
dit_status w_cross_kv(dit_ctx* c, const Run& R, const std::string& p, int blk) {
  const dit_config& g = c->cfg;
  const Plan& P = R.P; const WsLayout& L = R.L;
  const int d = g.hidden, Nt = P.Nt;
  if (!(gmax(c, p + ".xqnorm.g") <= 1024.f && gmax(c, p + ".xknorm.g") <= 1024.f))
    return fail(c, DIT_EUNSUPPORTED, "%s: cross-attention norm gains above 1024 do not fit the fp16 storage of its queries and keys", p.c_str());
  const bf16_t* cproj = R.at<bf16_t>(L.cproj);
  const bf16_t* cproj_lo = cproj + (size_t)Nt * d;
  float* kv32 = R.at<float>(L.act);
  run_gemm(c, {mk(cproj, d, Wm(c, p + ".xkv.w"), Wld(c, p + ".xkv.w"), Wv(c, p + ".xkv.b"), Nt, 2 * d, d, OUT_F32, kv32, 2 * d)});
  run_gemm(c, {mk(cproj_lo, d, Wm(c, p + ".xkv.w"), Wld(c, p + ".xkv.w"), nullptr, Nt, 2 * d, d, OUT_RESID_F32, kv32, 2 * d)});
  Scope sc(c, DIT_PROF_QKNORM, 0, 12.0 * Nt * d);
  launch_cross_kv_finish(c->stream, kv32, 2 * d, Nt, g.n_heads, g.head_dim, Wv(c, p + ".xknorm.g"),
                         R.at<bf16_t>(L.xk) + (size_t)blk * Nt * d, d, R.ip(P.o_src_of_col_x), P.Nvx_pad,
                         R.at<bf16_t>(L.vtx) + (size_t)blk * d * P.Nvx_pad, R.at<bf16_t>(L.vtlo) + (size_t)blk * d * P.Nvx_pad, P.Nvx_pad);
  return DIT_OK;
}

dit_status w_block(dit_ctx* c, const Run& R, const std::string& p, const float* base, int blk) {
  const dit_config& g = c->cfg;
  const Plan& P = R.P; const WsLayout& L = R.L;
  const int d = g.hidden, dff = g.mlp_hidden, Ni = P.Ni, Nt = P.Nt, e6 = 6 * d;
  float* x = R.at<float>(L.x);
  float* e = R.at<float>(L.modblk);
  bf16_t* h = R.at<bf16_t>(L.h); bf16_t* qkv = R.at<bf16_t>(L.qkv);
  bf16_t* q = R.at<bf16_t>(L.q); bf16_t* k = R.at<bf16_t>(L.k); bf16_t* vt = R.at<bf16_t>(L.vt);
  bf16_t* o = R.at<bf16_t>(L.o); bf16_t* act = R.at<bf16_t>(L.act);
  const int* rreq = R.ip(P.o_row_req_s);
  const float2* rope = (g.rope_axes[0] + g.rope_axes[1] + g.rope_axes[2]) > 0 ? R.at<float2>(L.rope) : nullptr;
  {
    Scope sc(c, DIT_PROF_OTHER, 0, 0);
    launch_add_rows(c->stream, base, L.MC, Wv(c, p + ".mod_table"), e, e6, P.n_req, e6);
  }
  {
    Scope sc(c, DIT_PROF_LNMOD, 0, 6.0 * Ni * d);
    launch_ln_modulate(c->stream, x, h, Ni, d, e, e + d, e6, rreq, nullptr, nullptr);
  }
  const bool fuse = c->taps.empty();          // see joint_block
  const float qs = attn_qscale(g.head_dim);
  GemmProblem pq = mk(h, d, Wm(c, p + ".qkv.w"), Wld(c, p + ".qkv.w"), Wv(c, p + ".qkv.b"), Ni, 3 * d, d, OUT_BF16, qkv, 3 * d);
  if (fuse) pq = with_vt(with_qknorm(pq, d, d, g.head_dim, Wv(c, p + ".qnorm.g"), Wv(c, p + ".knorm.g"), rope, nullptr, q, k, d, qs), vt, P.Nv_pad, R.ip(P.o_vtcol_s));
  run_gemm(c, {pq});
  if (!fuse) {
    Scope sc(c, DIT_PROF_QKNORM, 0, 12.0 * Ni * d);
    launch_qknorm_rope(c->stream, qkv, 3 * d, Ni, g.n_heads, g.head_dim, Wv(c, p + ".qnorm.g"), Wv(c, p + ".knorm.g"), rope, nullptr, q, k, d, d, 1,
                       -1, nullptr, nullptr, qs);
    launch_v_transpose(c->stream, qkv, 3 * d, 2 * d, g.n_heads, g.head_dim, R.ip(P.o_src_of_col), P.Nv_pad, vt, P.Nv_pad);
  }
  run_attention(c, R, q, d, k, d, vt, P.Nv_pad, o, d, R.ip(P.o_cu_joint), R.ip(P.o_cu_joint), R.ip(P.o_vt_off),
                (const AttnTile*)(R.ws + L.meta + P.o_tiles), (int)P.tiles.size(), nullptr, P.attn_flop,
                gmax(c, p + ".qnorm.g"), gmax(c, p + ".knorm.g"), nullptr, true);
  TAP(p + ".attn", o, Ni, d, 2, d);
  run_gemm(c, {mk(o, d, Wm(c, p + ".proj.w"), Wld(c, p + ".proj.w"), Wv(c, p + ".proj.b"), Ni, d, d, OUT_RESID_F32, x, d, e + 2 * d, e6, rreq)});
  TAP(p + ".x_attn", x, Ni, d, 4, d);
  // cross-attention to the projected condition
  {
    Scope sc(c, DIT_PROF_LNMOD, 0, 6.0 * Ni * d);
    launch_ln_modulate(c->stream, x, h, Ni, d, nullptr, nullptr, 0, nullptr, Wv(c, p + ".xnorm.g"), Wv(c, p + ".xnorm.b"));
  }
  // The cross-attention output enters the residual stream without a gate, so its rounding noise is
  // not damped as that of the gated branches is: queries and keys are stored as fp16 (both are
  // RMS-normalised, hence bounded) and the values go to the attention as two bf16 terms; keys and
  // values come from w_cross_kv below, once per call.
  // (The q/k norm is always the product's epilogue: there is no capture point between it and the attention.)
  GemmProblem pxq = with_qknorm(mk(h, d, Wm(c, p + ".xq.w"), Wld(c, p + ".xq.w"), Wv(c, p + ".xq.b"), Ni, d, d, OUT_BF16, qkv, d),
                                d, 0, g.head_dim, Wv(c, p + ".xqnorm.g"), nullptr, nullptr, nullptr, q, nullptr, d, qs);
  pxq.qk.f16 = 1;
  const bf16_t* xk = R.at<bf16_t>(L.xk) + (size_t)blk * Nt * d;
  const bf16_t* vtx = R.at<bf16_t>(L.vtx) + (size_t)blk * d * P.Nvx_pad;
  const bf16_t* vtlo = R.at<bf16_t>(L.vtlo) + (size_t)blk * d * P.Nvx_pad;
  run_gemm(c, {pxq});
  run_attention(c, R, q, d, xk, d, vtx, P.Nvx_pad, o, d, R.ip(P.o_cu_img), R.ip(P.o_cu_txt), R.ip(P.o_vtx_off),
                (const AttnTile*)(R.ws + L.meta + P.o_xtiles), (int)P.xtiles.size(), nullptr, P.xattn_flop,
                gmax(c, p + ".xqnorm.g"), gmax(c, p + ".xknorm.g"), vtlo);
  TAP(p + ".xattn", o, Ni, d, 2, d);
  run_gemm(c, {mk(o, d, Wm(c, p + ".xproj.w"), Wld(c, p + ".xproj.w"), Wv(c, p + ".xproj.b"), Ni, d, d, OUT_RESID_F32, x, d)});
  TAP(p + ".x_cross", x, Ni, d, 4, d);
  {
    Scope sc(c, DIT_PROF_LNMOD, 0, 6.0 * Ni * d);
    launch_ln_modulate(c->stream, x, h, Ni, d, e + 3 * d, e + 4 * d, e6, rreq, nullptr, nullptr);
  }
  run_gemm(c, {mk(h, d, Wm(c, p + ".mlp1.w"), Wld(c, p + ".mlp1.w"), Wv(c, p + ".mlp1.b"), Ni, dff, d, OUT_GELU_BF16, act, dff)});
  run_gemm(c, {mk(act, dff, Wm(c, p + ".mlp2.w"), Wld(c, p + ".mlp2.w"), Wv(c, p + ".mlp2.b"), Ni, d, dff, OUT_RESID_F32, x, d, e + 5 * d, e6, rreq)});
  TAP(p + ".x_out", x, Ni, d, 4, d);
  return DIT_OK;
}

// Host copy of max|g| of every norm-gain vector (a few KB, device to host, once after the
// weights changed): the attention launches use it to bound the logits.
dit_status ensure_gain_stats(dit_ctx* c) {
  if (c->gain_stats_valid) return DIT_OK;
  HIPCHK(c, hipStreamSynchronize(c->stream));      // pending weight writes on the context's stream
  std::vector<float> host;
  for (const TensorRec& t : c->tensors) {
    if (t.kind != 2) continue;
    const size_t n = (size_t)t.rows_in * t.cols_out;
    host.resize(n);
    HIPCHK(c, hipMemcpy(host.data(), c->weights + t.off, n * sizeof(float), hipMemcpyDeviceToHost));
    float m = 0.f;
    for (float v : host) m = std::isfinite(v) ? std::max(m, std::fabs(v)) : INFINITY;
    c->gain_absmax[t.name] = m;
  }
  c->gain_stats_valid = true;
  return DIT_OK;
}

dit_status run_sample(dit_ctx* c, int n_req, const dit_req* reqs, float* latents, const void* cond,
                      const float* sigmas /* [n_req][T+1] */, int T, int kind, float* v_out) {
  const dit_config& g = c->cfg;
  if (!c->weights || !c->ws) return fail(c, DIT_EINVAL, "dit_bind has not been called");
  if (!latents || !cond || !sigmas) return fail(c, DIT_EINVAL, "null latents, cond or sigmas");
  if (T <= 0) return fail(c, DIT_EINVAL, "T must be positive");
  if (kind != DIT_UPDATE_EULER && kind != DIT_UPDATE_DDIM) return fail(c, DIT_EINVAL, "unknown update_kind %d", kind);
  dit_status st = validate_reqs(c, n_req, reqs);
  if (st != DIT_OK) return st;
  // update coefficients (host, double)
  std::vector<float> sig((size_t)T * n_req), ca((size_t)T * n_req), cb((size_t)T * n_req);
  for (int r = 0; r < n_req; ++r)
    for (int j = 0; j < T; ++j) {
      const double sc = sigmas[(size_t)r * (T + 1) + j], sn = sigmas[(size_t)r * (T + 1) + j + 1];
      if (!(std::isfinite(sc) && std::isfinite(sn))) return fail(c, DIT_EINVAL, "non-finite sigma");
      double a, b;
      if (kind == DIT_UPDATE_EULER) { a = 1.0; b = sn - sc; }
      else {
        const double ac = 1.0 - sc * sc, an = 1.0 - sn * sn;
        if (ac <= 0.0 || an < 0.0) return fail(c, DIT_EINVAL, "DDIM needs |sigma_cur| < 1 and |sigma_next| <= 1");
        a = std::sqrt(an / ac);
        b = std::sqrt(1.0 - an) - std::sqrt(an * (1.0 - ac) / ac);
      }
      sig[(size_t)j * n_req + r] = (float)sc; ca[(size_t)j * n_req + r] = (float)a; cb[(size_t)j * n_req + r] = (float)b;
    }
  // plan (host side cached while the request list stays the same)
  bool same = c->plan_valid && c->plan.n_req == n_req &&
              memcmp(c->plan.reqs.data(), reqs, sizeof(dit_req) * n_req) == 0;
  if (!same) { build_plan(c, n_req, reqs, c->plan); c->plan_valid = true; }
  const Plan& P = c->plan;
  WsLayout L;
  layout_ws(c, P, T, L);
  if (L.total > c->ws_bytes)
    return fail(c, DIT_ENOMEM, "workspace has %zu bytes, this call needs %zu", c->ws_bytes, L.total);
  HIPCHK(c, hipSetDevice(c->device));
  if ((st = ensure_gain_stats(c)) != DIT_OK) return st;
  hipStream_t s = c->stream;
  Run R{c, P, L, c->ws};
  c->gemm_partial = (float*)(c->ws + L.partial);
  c->launch_refused = false;
  const int Rr = T * n_req;
  {
    // one host image [meta | sigma | a | b], matching the first regions of the workspace; it
    // lives in a ring slot until an event recorded after the copy has completed
    dit_ctx::Slot& sl = c->slots[c->next_slot];
    c->next_slot = (c->next_slot + 1) % 4;
    if (!sl.ev) HIPCHK(c, hipEventCreateWithFlags(&sl.ev, hipEventDisableTiming));
    if (sl.used) HIPCHK(c, hipEventSynchronize(sl.ev));
    const size_t head = L.feat;   // meta, sig, coef_a, coef_b are the regions before feat
    sl.buf.assign(head, 0);
    memcpy(sl.buf.data() + L.meta, P.meta.data(), P.meta_bytes);
    {   // conditioning matrices: entry 0, 1 = timestep MLP; 2.. = modulation matrices in the order of the columns of `mod`
      SkinnyMat* tb = (SkinnyMat*)(sl.buf.data() + L.meta + P.o_skinny);
      int nm = 0, off = 0;
      auto add = [&](const std::string& name, int n, bool cols) {
        tb[nm++] = SkinnyMat{Wm(c, name + ".w"), Wv(c, name + ".b"), n, Wld(c, name + ".w"), cols ? off : 0, 0};
        if (cols) off += n;
      };
      add("t_embed.1", g.hidden, false); add("t_embed.2", g.hidden, false);
      char nm_[64];
      if (g.family == DIT_FAMILY_W) add("t_proj", 6 * g.hidden, true);
      else {
        const char* pre = g.family == DIT_FAMILY_J ? "blk" : "dbl";
        for (int l = 0; l < g.n_blocks; ++l)
          for (const char* sn : {"txt", "img"}) { snprintf(nm_, sizeof nm_, "%s%d.%s.mod", pre, l, sn); add(nm_, 6 * g.hidden, true); }
        for (int l = 0; l < g.n_single; ++l) { snprintf(nm_, sizeof nm_, "sgl%d.mod", l); add(nm_, 3 * g.hidden, true); }
      }
      add("final.mod", 2 * g.hidden, true);
      c->n_skinny = nm;
    }
    memcpy(sl.buf.data() + L.sig, sig.data(), (size_t)Rr * 4);
    memcpy(sl.buf.data() + L.coef_a, ca.data(), (size_t)Rr * 4);
    memcpy(sl.buf.data() + L.coef_b, cb.data(), (size_t)Rr * 4);
    HIPCHK(c, hipMemcpyAsync(c->ws, sl.buf.data(), head, hipMemcpyHostToDevice, s));
    HIPCHK(c, hipEventRecord(sl.ev, s));
    sl.used = true;
  }

  const int d = g.hidden, Nt = P.Nt, Ni = P.Ni, MC = L.MC;
  const bool has_rope = (g.rope_axes[0] + g.rope_axes[1] + g.rope_axes[2]) > 0;
  float* mod = R.at<float>(L.mod);
  float* x = R.at<float>(L.x);
  const TokInfo* tok = (const TokInfo*)(c->ws + L.meta + P.o_tok);
  char nb[64];

  // ---- step-invariant work --------------------------------------------------------------
  {
    Scope sc(c, DIT_PROF_OTHER, 0, 0);
    launch_timestep_features(s, R.at<float>(L.sig), R.at<float>(L.feat), Rr);
    const SkinnyMat* mats = (const SkinnyMat*)(c->ws + L.meta + P.o_skinny);
    if (!launch_skinny(s, R.at<float>(L.feat), T_FREQ, mats, 1, d, R.at<float>(L.th1), d, Rr, T_FREQ, 0) ||
        !launch_skinny(s, R.at<float>(L.th1), d, mats + 1, 1, d, R.at<float>(L.vec), d, Rr, d, 1))
      return fail(c, DIT_ESHAPE, "hidden size %d: the conditioning products need a multiple of 8", d);
    const float* vec = R.at<float>(L.vec);
    int off = 0;
    // With many conditioning rows (steps x requests) the modulation products go to the MFMA
    // GEMM: SiLU(vec) enters as two bf16 terms, so the result agrees with the fp32 path to
    // ~1e-5 relative; with few rows the fp32 matrix-vector kernel is used.
    const bool big = Rr >= 16;      // (measured at hidden 1536: 16 rows take 41.1 ms per 16-step sample this way, 42.2 ms the other)
    if (big) launch_silu_split(s, vec, R.at<bf16_t>(L.mhi), R.at<bf16_t>(L.mlo), (long long)Rr * d);
    else      // one launch for every modulation matrix: each is read once, all rows at a time
      launch_skinny(s, vec, d, mats + 2, c->n_skinny - 2, 6 * d, mod, MC, Rr, d, 1);
    auto modv = [&](const std::string& name, int n) {
      if (big) {
        run_gemm(c, {mk(R.at<bf16_t>(L.mhi), d, Wm(c, name + ".w"), Wld(c, name + ".w"), Wv(c, name + ".b"), Rr, n, d, OUT_F32, mod + off, MC)});
        run_gemm(c, {mk(R.at<bf16_t>(L.mlo), d, Wm(c, name + ".w"), Wld(c, name + ".w"), nullptr, Rr, n, d, OUT_RESID_F32, mod + off, MC)});
      }
      off += n;
    };
    if (g.family == DIT_FAMILY_W) modv("t_proj", 6 * d);
    else {
      const char* pre = g.family == DIT_FAMILY_J ? "blk" : "dbl";
      for (int l = 0; l < g.n_blocks; ++l)
        for (const char* sn : {"txt", "img"}) { snprintf(nb, sizeof nb, "%s%d.%s.mod", pre, l, sn); modv(nb, 6 * d); }
      for (int l = 0; l < g.n_single; ++l) { snprintf(nb, sizeof nb, "sgl%d.mod", l); modv(nb, 3 * d); }
    }
    modv("final.mod", 2 * d);
    // the QKV epilogue writes only the columns of real tokens: the pad columns of every request's
    // transposed values (up to the next multiple of 64) are zeroed here, once for all steps and blocks
    launch_fill_u16(s, R.at<bf16_t>(L.vt), (long long)d * P.Nv_pad, 0);
    if (has_rope)
      launch_rope_table(s, tok, R.ip(P.o_tok_of_row), P.Nj, g.head_dim, g.rope_axes[0], g.rope_axes[1], g.rope_axes[2], g.rope_theta, R.at<float2>(L.rope));
  }
  // condition projection
  run_gemm(c, {mk((const bf16_t*)cond, g.cond_dim, Wm(c, "c_embed.w"), Wld(c, "c_embed.w"), Wv(c, "c_embed.b"), Nt, d, g.cond_dim, OUT_F32, R.at<float>(L.xt0), d)});
  if (!P.has_txt_stream) {      // family W: the cross-attention reads it as two bf16 terms
    Scope sc(c, DIT_PROF_OTHER, 0, 0);
    launch_silu_split(s, R.at<float>(L.xt0), R.at<bf16_t>(L.cproj), R.at<bf16_t>(L.cproj) + (size_t)Nt * d, (long long)Nt * d, 0);
  }
  if (g.family == DIT_FAMILY_W)
    for (int l = 0; l < g.n_blocks; ++l) {
      snprintf(nb, sizeof nb, "blk%d", l);
      if ((st = w_cross_kv(c, R, nb, l)) != DIT_OK) return st;
    }

  const int soff_img = P.has_txt_stream ? Nt : 0;
  float* x_img = x + (size_t)soff_img * d;
  for (int step = 0; step < T; ++step) {
    const float* mstep = mod + (size_t)step * n_req * MC;
    // ---- embed ---------------------------------------------------------------------------
    {
      Scope sc(c, DIT_PROF_OTHER, 0, 0);
      launch_patchify(s, latents, (const long long*)(c->ws + L.meta + P.o_lat_off), (const int4*)(c->ws + L.meta + P.o_req_dims),
                      tok, Ni, g.latent_ch, g.patch_t, g.patch_h, g.patch_w, R.at<bf16_t>(L.patch),
                      R.at<bf16_t>(L.patch) + (size_t)Ni * L.ldp, L.ldp);
      if (P.has_txt_stream) launch_copy_rows_f32(s, R.at<float>(L.xt0), nullptr, x, nullptr, Nt, d);
    }
    // The latent enters as two bf16 terms (hi + lo) so that the embedding sees it to ~16 bits:
    // with small weights the model output is dominated by this path and by the final layer.
    run_gemm(c, {mk(R.at<bf16_t>(L.patch), L.ldp, Wm(c, "x_embed.w"), Wld(c, "x_embed.w"), Wv(c, "x_embed.b"), Ni, d, L.ldp, OUT_F32, x_img, d)});
    run_gemm(c, {mk(R.at<bf16_t>(L.patch) + (size_t)Ni * L.ldp, L.ldp, Wm(c, "x_embed.w"), Wld(c, "x_embed.w"), nullptr, Ni, d, L.ldp, OUT_RESID_F32, x_img, d)});
    if (g.family == DIT_FAMILY_J) {
      Scope sc(c, DIT_PROF_OTHER, 0, 0);
      launch_add_pe(s, x_img, tok, Ni, d);
    }
    if (P.has_txt_stream) TAP("x_txt0", x, Nt, d, 4, d);
    TAP("x_img0", x_img, Ni, d, 4, d);
    // ---- blocks --------------------------------------------------------------------------
    int off = 0;
    if (g.family == DIT_FAMILY_J || g.family == DIT_FAMILY_F) {
      const char* pre = g.family == DIT_FAMILY_J ? "blk" : "dbl";
      for (int l = 0; l < g.n_blocks; ++l, off += 12 * d) {
        snprintf(nb, sizeof nb, "%s%d", pre, l);
        if ((st = joint_block(c, R, nb, mstep, off)) != DIT_OK) return st;
      }
      if (g.n_single > 0) {
        { Scope sc(c, DIT_PROF_OTHER, 0, 0); launch_copy_rows_f32(s, x, nullptr, R.at<float>(L.xj), R.ip(P.o_s2j), P.Ns, d); }
        for (int l = 0; l < g.n_single; ++l, off += 3 * d) {
          snprintf(nb, sizeof nb, "sgl%d", l);
          if ((st = single_block(c, R, nb, mstep, off)) != DIT_OK) return st;
        }
        { Scope sc(c, DIT_PROF_OTHER, 0, 0); launch_copy_rows_f32(s, R.at<float>(L.xj), R.ip(P.o_s2j), x, nullptr, P.Ns, d); }
      }
    } else {
      off = 6 * d;
      for (int l = 0; l < g.n_blocks; ++l) {
        snprintf(nb, sizeof nb, "blk%d", l);
        if ((st = w_block(c, R, nb, mstep, l)) != DIT_OK) return st;
      }
    }
    // ---- final layer + latent update -----------------------------------------------------
    const float* mf = mstep + off;
    bf16_t* h = R.at<bf16_t>(L.h);
    {
      Scope sc(c, DIT_PROF_LNMOD, 0, 6.0 * Ni * d);
      launch_ln_modulate(s, x_img, h, Ni, d, mf, mf + d, MC, R.ip(P.o_row_req_s) + soff_img, nullptr, nullptr,
                         R.at<bf16_t>(L.o));     // second term in the (free) attention-output buffer
    }
    run_gemm(c, {mk(h, d, Wm(c, "final.w"), Wld(c, "final.w"), Wv(c, "final.b"), Ni, c->pdim, d, OUT_F32, R.at<float>(L.yfin), L.ldy)});
    run_gemm(c, {mk(R.at<bf16_t>(L.o), d, Wm(c, "final.w"), Wld(c, "final.w"), nullptr, Ni, c->pdim, d, OUT_RESID_F32, R.at<float>(L.yfin), L.ldy)});
    TAP("final", R.at<float>(L.yfin), Ni, c->pdim, 4, L.ldy);
    {
      Scope sc(c, DIT_PROF_UPDATE, 0, 12.0 * P.lat_total);
      launch_unpatchify_update(s, latents, v_out, R.at<float>(L.yfin), L.ldy, (const long long*)(c->ws + L.meta + P.o_lat_off),
                               (const int4*)(c->ws + L.meta + P.o_req_dims), R.ip(P.o_cu_img),
                               R.at<float>(L.coef_a) + (size_t)step * n_req, R.at<float>(L.coef_b) + (size_t)step * n_req,
                               n_req, P.lat_total, g.latent_ch, g.patch_t, g.patch_h, g.patch_w);
    }
  }
  HIPCHK(c, hipGetLastError());
  if (c->launch_refused) return fail(c, DIT_ESHAPE, "a matrix product of this call exceeds the GEMM kernels' 4 GiB operand limit");
  return DIT_OK;
}

}  // namespace

// Split-K scratch that lives in the library's own device image, for callers that may not
// allocate: one array per GPU the library runs on (every device loads its own copy of the
// code object), held until the process ends.  The name below is a host-side stand-in; the
// device address is looked up once per device and only that pointer is ever handed to
// kernels.
static __device__ __align__(256) unsigned char scratch[DIT_STATIC_SCRATCH_BYTES];
static std::atomic<unsigned char*> scratch_ptr[32];    // per device: address of its copy


// =======================================================================================
// C ABI
// =======================================================================================
extern "C" {

dit_status dit_create(const dit_config* cfg, int device, void* hip_stream, dit_ctx** out) {
  if (out) *out = nullptr;
  if (!cfg || !out) return DIT_EINVAL;
  const dit_config& g = *cfg;
  if (g.family < 0 || g.family > 2) return DIT_EINVAL;
  if (g.n_blocks < 0 || g.n_single < 0 || (g.family != DIT_FAMILY_F && g.n_single != 0)) return DIT_ESHAPE;
  if (g.hidden <= 0 || g.hidden % 256 || g.hidden > 5120) return DIT_ESHAPE;
  if (g.n_heads <= 0 || (g.head_dim != 64 && g.head_dim != 128) || g.hidden != g.n_heads * g.head_dim) return DIT_ESHAPE;
  if (g.mlp_hidden <= 0 || g.mlp_hidden % 256) return DIT_ESHAPE;
  if (g.latent_ch <= 0 || g.patch_t <= 0 || g.patch_h <= 0 || g.patch_w <= 0) return DIT_ESHAPE;
  if (g.cond_dim <= 0 || g.cond_dim % 64) return DIT_ESHAPE;
  const int rs = g.rope_axes[0] + g.rope_axes[1] + g.rope_axes[2];
  for (int a = 0; a < 3; ++a)
    if (g.rope_axes[a] < 0 || g.rope_axes[a] % 2) return DIT_ESHAPE;
  if (rs != 0 && rs != g.head_dim) return DIT_ESHAPE;
  if (rs != 0 && !(g.rope_theta > 1.0f)) return DIT_EINVAL;
  if (g.family == DIT_FAMILY_J && rs != 0) return DIT_EUNSUPPORTED;
  if (g.act_dtype != DIT_ACT_F32 && g.act_dtype != DIT_ACT_BF16) return DIT_EINVAL;
  if (g.act_dtype == DIT_ACT_F32) return DIT_EUNSUPPORTED;      // only bf16 activation storage is built
  if ((long long)g.latent_ch * g.patch_t * g.patch_h * g.patch_w > 1024) return DIT_ESHAPE;
  dit_ctx* c = new (std::nothrow) dit_ctx();
  if (!c) return DIT_ENOMEM;
  c->cfg = g; c->device = device; c->stream = (hipStream_t)hip_stream;
  c->pdim = g.latent_ch * g.patch_t * g.patch_h * g.patch_w;
  build_table(c);
  *out = c;
  return DIT_OK;
}

void dit_destroy(dit_ctx* c) {
  if (!c) return;
  for (hipEvent_t e : c->ev_pool) (void)hipEventDestroy(e);
  for (auto& sl : c->slots) if (sl.ev) (void)hipEventDestroy(sl.ev);
  delete c;
}

dit_status dit_set_stream(dit_ctx* c, void* s) {
  if (!c) return DIT_EINVAL;
  c->stream = (hipStream_t)s;
  return DIT_OK;
}

const char* dit_last_error(const dit_ctx* c) { return c ? c->err.c_str() : "null context"; }

size_t dit_weight_bytes(const dit_ctx* c) { return c ? c->weight_bytes : 0; }

size_t dit_workspace_bytes(const dit_ctx* c, int n_req, const dit_req* reqs, int max_steps) {
  if (!c || max_steps <= 0 || validate_reqs(c, n_req, reqs) != DIT_OK) return 0;
  Plan P; WsLayout L;
  build_plan(c, n_req, reqs, P);
  layout_ws(c, P, max_steps, L);
  return L.total;
}

dit_status dit_attention_plan(const dit_ctx* c, int n_req, const dit_req* reqs, int out[4]) {
  if (!c || !out) return DIT_EINVAL;
  if (validate_reqs(c, n_req, reqs) != DIT_OK) return DIT_ESHAPE;
  Plan P;
  build_plan(c, n_req, reqs, P);
  out[0] = P.qb; out[1] = (int)P.tiles.size(); out[2] = P.split_slots; out[3] = P.split_parts;
  return DIT_OK;
}

dit_status dit_bind(dit_ctx* c, void* w, size_t wb, void* ws, size_t wsb) {
  if (!c) return DIT_EINVAL;
  if (!w || !ws) return fail(c, DIT_EINVAL, "null buffer");
  if (((uintptr_t)w & 255) || ((uintptr_t)ws & 255)) return fail(c, DIT_EINVAL, "buffers must be 256-byte aligned");
  if (wb < c->weight_bytes) return fail(c, DIT_ENOMEM, "weight arena has %zu bytes, needs %zu", wb, c->weight_bytes);
  c->weights = (unsigned char*)w; c->ws = (unsigned char*)ws; c->ws_bytes = wsb;
  c->gain_stats_valid = false;
  return DIT_OK;
}

static uint64_t fnv1a64(const std::string& s) {
  uint64_t h = 0xCBF29CE484222325ull;
  for (unsigned char ch : s) { h ^= ch; h *= 0x100000001B3ull; }
  return h;
}
static uint64_t mix64(uint64_t x) {
  uint64_t z = x + 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

dit_status dit_init_weights(dit_ctx* c, uint64_t seed, float std) {
  if (!c) return DIT_EINVAL;
  if (!c->weights) return fail(c, DIT_EINVAL, "dit_bind has not been called");
  if (!(std >= 0.f) || !std::isfinite(std)) return fail(c, DIT_EINVAL, "std must be finite and non-negative");
  HIPCHK(c, hipSetDevice(c->device));
  c->gain_stats_valid = false;
  HIPCHK(c, hipMemsetAsync(c->weights, 0, c->weight_bytes, c->stream));
  for (const TensorRec& t : c->tensors) {
    const uint64_t key = mix64(seed ^ (fnv1a64(t.name) * 0x9E3779B97F4A7C15ull));
    if (t.kind == 0) launch_init_matrix(c->stream, (bf16_t*)(c->weights + t.off), t.cols_out, t.rows_in, t.ld, key, std);
    else if (t.kind == 3) launch_init_table_f32(c->stream, (float*)(c->weights + t.off), (long long)t.rows_in * t.cols_out, key, std);
    else if (t.kind == 2) launch_fill_f32(c->stream, (float*)(c->weights + t.off), t.cols_out, 1.0f);
  }
  HIPCHK(c, hipGetLastError());
  return DIT_OK;
}

int dit_tensor_count(const dit_ctx* c) { return c ? (int)c->tensors.size() : 0; }

dit_status dit_tensor_info(const dit_ctx* c, int i, char* name, size_t len, int* rows_in, int* cols_out, int* kind) {
  if (!c) return DIT_EINVAL;
  if (i < 0 || i >= (int)c->tensors.size()) return fail(c, DIT_ENOTFOUND, "tensor index %d out of range", i);
  const TensorRec& t = c->tensors[i];
  if (name && len) { strncpy(name, t.name.c_str(), len - 1); name[len - 1] = 0; }
  if (rows_in) *rows_in = t.rows_in;
  if (cols_out) *cols_out = t.cols_out;
  if (kind) *kind = t.kind;
  return DIT_OK;
}

static uint16_t host_f2bf(float f) {
  uint32_t u; memcpy(&u, &f, 4);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

dit_status dit_set_tensor(dit_ctx* c, const char* name, const float* src, size_t n) {
  if (!c || !name || !src) return DIT_EINVAL;
  if (!c->weights) return fail(c, DIT_EINVAL, "dit_bind has not been called");
  const TensorRec* t = find(c, name);
  if (!t) return fail(c, DIT_ENOTFOUND, "no tensor named %s", name);
  if (n != (size_t)t->rows_in * t->cols_out) return fail(c, DIT_ESHAPE, "%s has %d x %d elements", name, t->rows_in, t->cols_out);
  HIPCHK(c, hipSetDevice(c->device));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  c->gain_stats_valid = false;
  if (t->kind == 0) {
    std::vector<uint16_t> buf((size_t)t->rows_pad * t->ld, 0);   // pads are written as zeros
    for (int i = 0; i < t->rows_in; ++i)
      for (int o = 0; o < t->cols_out; ++o) buf[(size_t)o * t->ld + i] = host_f2bf(src[(size_t)i * t->cols_out + o]);
    HIPCHK(c, hipMemcpy(c->weights + t->off, buf.data(), buf.size() * 2, hipMemcpyHostToDevice));
  } else {
    HIPCHK(c, hipMemcpy(c->weights + t->off, src, n * 4, hipMemcpyHostToDevice));
  }
  return DIT_OK;
}

dit_status dit_get_tensor(dit_ctx* c, const char* name, float* dst, size_t n) {
  if (!c || !name || !dst) return DIT_EINVAL;
  if (!c->weights) return fail(c, DIT_EINVAL, "dit_bind has not been called");
  const TensorRec* t = find(c, name);
  if (!t) return fail(c, DIT_ENOTFOUND, "no tensor named %s", name);
  if (n != (size_t)t->rows_in * t->cols_out) return fail(c, DIT_ESHAPE, "%s has %d x %d elements", name, t->rows_in, t->cols_out);
  HIPCHK(c, hipSetDevice(c->device));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  if (t->kind == 0) {
    std::vector<uint16_t> buf((size_t)t->cols_out * t->ld);
    HIPCHK(c, hipMemcpy(buf.data(), c->weights + t->off, buf.size() * 2, hipMemcpyDeviceToHost));
    for (int i = 0; i < t->rows_in; ++i)
      for (int o = 0; o < t->cols_out; ++o) {
        uint32_t u = (uint32_t)buf[(size_t)o * t->ld + i] << 16;
        memcpy(&dst[(size_t)i * t->cols_out + o], &u, 4);
      }
  } else {
    HIPCHK(c, hipMemcpy(dst, c->weights + t->off, n * 4, hipMemcpyDeviceToHost));
  }
  return DIT_OK;
}

dit_status dit_denoise_step(dit_ctx* c, int n_req, const dit_req* reqs, float* latents, const void* cond,
                            const float* sigma_cur, const float* sigma_next, int kind, float* v_out) {
  if (!c) return DIT_EINVAL;
  if (!sigma_cur || !sigma_next) return fail(c, DIT_EINVAL, "null sigma arrays");
  if (n_req <= 0) return fail(c, DIT_EINVAL, "n_req must be positive");
  std::vector<float> sg((size_t)n_req * 2);
  for (int r = 0; r < n_req; ++r) { sg[2 * r] = sigma_cur[r]; sg[2 * r + 1] = sigma_next[r]; }
  return run_sample(c, n_req, reqs, latents, cond, sg.data(), 1, kind, v_out);
}

dit_status dit_sample(dit_ctx* c, int n_req, const dit_req* reqs, float* latents, const void* cond,
                      const float* sigmas, int T, int kind) {
  if (!c) return DIT_EINVAL;
  return run_sample(c, n_req, reqs, latents, cond, sigmas, T, kind, nullptr);
}

dit_status dit_set_tap(dit_ctx* c, const char* point, void* dst, size_t bytes) {
  if (!c || !point || !dst) return DIT_EINVAL;
  c->taps[point] = Tap{dst, bytes, 0, 0, 0};
  return DIT_OK;
}
dit_status dit_tap_info(const dit_ctx* c, const char* point, int* rows, int* cols, int* elem) {
  if (!c || !point) return DIT_EINVAL;
  auto it = c->taps.find(point);
  if (it == c->taps.end()) return fail(c, DIT_ENOTFOUND, "no tap named %s", point);
  if (rows) *rows = it->second.rows;
  if (cols) *cols = it->second.cols;
  if (elem) *elem = it->second.elem;
  return DIT_OK;
}
void dit_clear_taps(dit_ctx* c) { if (c) c->taps.clear(); }

dit_status dit_profile_enable(dit_ctx* c, int on) {
  if (!c) return DIT_EINVAL;
  if (on) {
    HIPCHK(c, hipStreamSynchronize(c->stream));
    for (hipEvent_t e : c->ev_pool) (void)hipEventDestroy(e);
    c->ev_pool.clear(); c->ev_recs.clear();
    for (int k = 0; k < DIT_PROF_NCLASS; ++k) c->prof_flop[k] = c->prof_bytes[k] = 0;
  }
  c->prof = on != 0;
  return DIT_OK;
}

dit_status dit_profile_read(dit_ctx* c, int klass, double* total_ms, long long* launches, double* flop, double* bytes) {
  if (!c) return DIT_EINVAL;
  if (klass < 0 || klass >= DIT_PROF_NCLASS) return fail(c, DIT_EINVAL, "bad class %d", klass);
  HIPCHK(c, hipStreamSynchronize(c->stream));
  double ms = 0; long long n = 0;
  for (size_t i = 0; i < c->ev_recs.size(); ++i) {
    if (c->ev_recs[i].klass != klass) continue;
    float t = 0;
    HIPCHK(c, hipEventElapsedTime(&t, c->ev_pool[2 * i], c->ev_pool[2 * i + 1]));
    ms += t; ++n;
  }
  if (total_ms) *total_ms = ms;
  if (launches) *launches = n;
  if (flop) *flop = c->prof_flop[klass];
  if (bytes) *bytes = c->prof_bytes[klass];
  return DIT_OK;
}

// ---- single operations ----------------------------------------------------------------

dit_status dit_op_gemm(void* stream, const void* A, int lda, const void* W, int ldw, const float* bias, int M, int N,
                       int K, int out_kind, void* out, int ldc, const float* gate, int gate_stride,
                       const int* row_req) {
  if (!A || !W || !out) return DIT_EINVAL;
  if (M < 0 || N < 0 || K <= 0 || K % 64 || lda < K || ldw < K || ldc < N) return DIT_ESHAPE;
  if (lda % 8 || ldw % 8) return DIT_ESHAPE;
  if (out_kind < 0 || out_kind > 3) return DIT_EINVAL;
  if (ldc % ((out_kind == 1 || out_kind == 3) ? 4 : 8) || ((uintptr_t)out & 15)) return DIT_ESHAPE;
  if (M == 0 || N == 0) return DIT_OK;
  GemmBatch b; b.n = 1; b.total_tiles = 0;
  b.p[0] = mk((const bf16_t*)A, lda, (const bf16_t*)W, ldw, bias, M, N, K, out_kind, out, ldc, gate, gate_stride, row_req);
  if (launch_gemm((hipStream_t)stream, b, 0) < 0) return DIT_ESHAPE;
  return hipGetLastError() == hipSuccess ? DIT_OK : DIT_EDEVICE;
}

dit_status dit_op_gemm_qknorm(void* stream, const void* A, int lda, const void* W, int ldw, const float* bias, int M,
                              int N, int K, void* out, int ldc, int nq, int nk, int head_dim, const float* qgain,
                              const float* kgain, const float* rope, const int* dst_row, void* qo, void* ko,
                              int ldo, float qscale) {
  if (!A || !W || !out) return DIT_EINVAL;
  if (M <= 0 || N <= 0 || K <= 0 || K % 64 || lda < K || ldw < K || ldc < N) return DIT_ESHAPE;
  if (lda % 8 || ldw % 8 || ldc % 8 || N % 8 || ((uintptr_t)out & 15)) return DIT_ESHAPE;
  if (head_dim != 64 && head_dim != 128) return DIT_ESHAPE;
  if (nq < 0 || nk < 0 || nq % 256 || nk % 256 || nq + nk > N || nq + nk == 0) return DIT_ESHAPE;
  if ((nq && (!qo || !qgain)) || (nk && (!ko || !kgain))) return DIT_EINVAL;
  if (ldo % 8 || ldo < std::max(nq, nk) || ((uintptr_t)qo & 15) || ((uintptr_t)ko & 15)) return DIT_ESHAPE;
  GemmBatch b; b.n = 1; b.total_tiles = 0;
  b.p[0] = with_qknorm(mk((const bf16_t*)A, lda, (const bf16_t*)W, ldw, bias, M, N, K, OUT_BF16, out, ldc), nq, nk,
                       head_dim, qgain, kgain, (const float2*)rope, dst_row, (bf16_t*)qo, (bf16_t*)ko, ldo, qscale);
  if (launch_gemm((hipStream_t)stream, b, 0) < 0) return DIT_ESHAPE;
  return hipGetLastError() == hipSuccess ? DIT_OK : DIT_EDEVICE;
}

dit_status dit_op_gemm_splitk(void* stream, const void* A, int lda, const void* W, int ldw, const float* bias, int M,
                              int N, int K, int out_kind, void* out, int ldc, const float* gate, int gate_stride,
                              const int* row_req, int splits, void* work, size_t work_bytes) {
  if (!A || !W || !out || !work) return DIT_EINVAL;
  if (M <= 0 || N <= 0 || K <= 0 || K % 64 || lda < K || ldw < K || ldc < N) return DIT_ESHAPE;
  if (lda % 8 || ldw % 8) return DIT_ESHAPE;
  if (out_kind < 0 || out_kind > 3) return DIT_EINVAL;
  if (ldc % ((out_kind == 1 || out_kind == 3) ? 4 : 8) || ((uintptr_t)out & 15) || ((uintptr_t)work & 15)) return DIT_ESHAPE;
  if (splits < 1 || splits > K / 64) return DIT_ESHAPE;
  const size_t tiles = (size_t)((M + 127) / 128) * ((N + 127) / 128);
  if (work_bytes < tiles * splits * (128 * 128 * 4)) return DIT_ENOMEM;
  GemmBatch b; b.n = 1; b.total_tiles = 0;
  b.p[0] = mk((const bf16_t*)A, lda, (const bf16_t*)W, ldw, bias, M, N, K, out_kind, out, ldc, gate, gate_stride, row_req);
  b.splits = splits; b.partial = (float*)work; b.partial_bytes = work_bytes;
  if (launch_gemm((hipStream_t)stream, b, 40128128) < 0) return DIT_ESHAPE;
  return hipGetLastError() == hipSuccess ? DIT_OK : DIT_EDEVICE;
}

dit_status dit_op_gemm_splitk_static(void* stream, const void* A, int lda, const void* W, int ldw, const float* bias,
                                     int M, int N, int K, int out_kind, void* out, int ldc, const float* gate,
                                     int gate_stride, const int* row_req, int splits) {
  if (!A || !W || !out) return DIT_EINVAL;
  if (M <= 0 || N <= 0 || K <= 0 || K % 64 || lda < K || ldw < K || ldc < N) return DIT_ESHAPE;
  if (lda % 8 || ldw % 8) return DIT_ESHAPE;
  if (out_kind < 0 || out_kind > 3) return DIT_EINVAL;
  if (ldc % ((out_kind == 1 || out_kind == 3) ? 4 : 8) || ((uintptr_t)out & 15)) return DIT_ESHAPE;
  if (splits < 1 || splits > K / 64) return DIT_ESHAPE;
  const size_t tiles = (size_t)((M + 127) / 128) * ((N + 127) / 128);
  if (tiles * splits * (128 * 128 * 4) > (size_t)DIT_STATIC_SCRATCH_BYTES) return DIT_ENOMEM;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 32) return DIT_EDEVICE;
  unsigned char* ptr = scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {      // first call on this device (it is the current one): where its copy of the array lives
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return DIT_EDEVICE;
    ptr = (unsigned char*)p;
    scratch_ptr[dev].store(ptr, std::memory_order_release);
  }
  GemmBatch b; b.n = 1; b.total_tiles = 0;
  b.p[0] = mk((const bf16_t*)A, lda, (const bf16_t*)W, ldw, bias, M, N, K, out_kind, out, ldc, gate, gate_stride, row_req);
  // every partial tile the reduction reads is written in full by the product kernel of the
  // same call, so nothing of the previous call's contents has to be cleared
  b.splits = splits; b.partial = (float*)ptr; b.partial_bytes = DIT_STATIC_SCRATCH_BYTES;
  if (launch_gemm((hipStream_t)stream, b, 40128128) < 0) return DIT_ESHAPE;
  return hipGetLastError() == hipSuccess ? DIT_OK : DIT_EDEVICE;
}

dit_status dit_op_gemm_variant(void* stream, const void* A, int lda, const void* W, int ldw, const float* bias, int M,
                               int N, int K, int out_kind, void* out, int ldc, int variant) {
  if (!A || !W || !out) return DIT_EINVAL;
  if (M <= 0 || N <= 0 || K <= 0 || K % 64 || lda < K || ldw < K || ldc < N) return DIT_ESHAPE;
  if (out_kind < 0 || out_kind > 2) return DIT_EINVAL;
  if (lda % 8 || ldw % 8 || ldc % (out_kind == 1 ? 4 : 8) || ((uintptr_t)out & 15)) return DIT_ESHAPE;
  GemmBatch b; b.n = 1; b.total_tiles = 0;
  b.p[0] = mk((const bf16_t*)A, lda, (const bf16_t*)W, ldw, bias, M, N, K, out_kind, out, ldc);
  if (launch_gemm((hipStream_t)stream, b, variant) < 0) return DIT_ESHAPE;
  return hipGetLastError() == hipSuccess ? DIT_OK : DIT_EDEVICE;
}

size_t dit_op_attention_work_bytes(int n_seg, const int* cu_q) {
  if (n_seg <= 0 || !cu_q) return 0;
  size_t tiles = 0;
  for (int s = 0; s < n_seg; ++s) tiles += (size_t)(cu_q[s + 1] - cu_q[s] + 127) / 128;   // upper bound for either tile size
  return rup((size_t)(n_seg + 1) * 4, 256) * 2 + rup((size_t)n_seg * 4, 256) + rup(tiles * sizeof(AttnTile), 256);
}

dit_status dit_op_attention(void* stream, const void* q, int ldq, const void* k, int ldk, const void* vt, int ldvt,
                            void* o, int ldo, int n_heads, int head_dim, int n_seg, const int* cu_q, const int* cu_k,
                            const int* vt_off, void* work, size_t work_bytes, int q_prescaled, float logit_bound) {
  if (!q || !k || !vt || !o || !cu_q || !cu_k || !vt_off || !work) return DIT_EINVAL;
  if (n_seg <= 0 || n_heads <= 0 || (head_dim != 64 && head_dim != 128)) return DIT_ESHAPE;
  const int d = n_heads * head_dim;
  if (ldq < d || ldk < d || ldo < d || ldq % 8 || ldk % 8 || ldo % 4 || ldvt % 64) return DIT_ESHAPE;
  std::vector<AttnTile> tiles;
  int longest = 0;
  for (int s = 0; s < n_seg; ++s) longest = std::max(longest, cu_k[s + 1] - cu_k[s]);
  const int qb = attn_q_per_tile(longest, head_dim);
  for (int s = 0; s < n_seg; ++s) {
    const int nq = cu_q[s + 1] - cu_q[s], nk = cu_k[s + 1] - cu_k[s];
    if (nq < 0 || nk <= 0 || vt_off[s] % 64 || vt_off[s] < 0) return DIT_ESHAPE;
    if (vt_off[s] + (int)rup(nk, 64) > ldvt) return DIT_ESHAPE;
    for (int q0 = 0; q0 < nq; q0 += qb) tiles.push_back(AttnTile{s, q0});
  }
  if (work_bytes < dit_op_attention_work_bytes(n_seg, cu_q)) return DIT_ENOMEM;
  std::stable_sort(tiles.begin(), tiles.end(), [&](const AttnTile& a, const AttnTile& b) {
    return cu_k[a.seg + 1] - cu_k[a.seg] > cu_k[b.seg + 1] - cu_k[b.seg];
  });
  hipStream_t s = (hipStream_t)stream;
  unsigned char* w = (unsigned char*)work;
  const size_t cu_b = rup((size_t)(n_seg + 1) * 4, 256), vo_b = rup((size_t)n_seg * 4, 256);
  if (hipMemcpyAsync(w, cu_q, (size_t)(n_seg + 1) * 4, hipMemcpyHostToDevice, s) != hipSuccess) return DIT_EDEVICE;
  if (hipMemcpyAsync(w + cu_b, cu_k, (size_t)(n_seg + 1) * 4, hipMemcpyHostToDevice, s) != hipSuccess) return DIT_EDEVICE;
  if (hipMemcpyAsync(w + 2 * cu_b, vt_off, (size_t)n_seg * 4, hipMemcpyHostToDevice, s) != hipSuccess) return DIT_EDEVICE;
  if (!tiles.empty() &&
      hipMemcpyAsync(w + 2 * cu_b + vo_b, tiles.data(), tiles.size() * sizeof(AttnTile), hipMemcpyHostToDevice, s) != hipSuccess)
    return DIT_EDEVICE;
  AttnArgs a;
  a.q = (const bf16_t*)q; a.ldq = ldq; a.k = (const bf16_t*)k; a.ldk = ldk; a.vt = (const bf16_t*)vt; a.ldvt = ldvt;
  a.o = (bf16_t*)o; a.ldo = ldo; a.n_heads = n_heads; a.head_dim = head_dim;
  a.cu_q = (const int*)w; a.cu_k = (const int*)(w + cu_b); a.vt_off = (const int*)(w + 2 * cu_b);
  a.tiles = (const AttnTile*)(w + 2 * cu_b + vo_b); a.n_tiles = (int)tiles.size(); a.o_row_map = nullptr;
  a.q_per_tile = qb;
  a.scale_log2 = attn_qscale(head_dim);
  a.mode = !q_prescaled ? 0 : (logit_bound > 0.f && logit_bound <= 60.f) ? 2 : 1;
  launch_attention(s, a);
  return hipGetLastError() == hipSuccess ? DIT_OK : DIT_EDEVICE;
}

dit_status dit_op_ln_modulate(void* stream, const float* x, void* y, int M, int d, const float* shift,
                              const float* scale, int mod_stride, const int* row_req) {
  if (!x || !y || !shift || !scale) return DIT_EINVAL;
  if (M < 0 || d <= 0 || d % 256 || d > 5120) return DIT_ESHAPE;
  launch_ln_modulate((hipStream_t)stream, x, (bf16_t*)y, M, d, shift, scale, mod_stride, row_req, nullptr, nullptr, nullptr);
  return hipGetLastError() == hipSuccess ? DIT_OK : DIT_EDEVICE;
}

dit_status dit_op_latent_update(void* stream, float* x, const float* v, long long n, float a, float b) {
  if (!x || !v) return DIT_EINVAL;
  if (n < 0) return DIT_ESHAPE;
  launch_latent_update((hipStream_t)stream, x, v, n, a, b);
  return hipGetLastError() == hipSuccess ? DIT_OK : DIT_EDEVICE;
}

}  // extern "C"
