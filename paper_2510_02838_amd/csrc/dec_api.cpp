// Host runtime of the Decode stage (AutoencoderKL-style convolutional decoder): tensor table,
// workspace layout and the launch sequence of one forward pass.  Every arithmetic step runs in
// the kernels of gemm.hip (convolutions as products), elementwise.hip and decoder.hip.
#include "../../include/decoder.h"
#include "dit_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <string>
#include <unordered_map>
#include <vector>

using namespace dit;

namespace {
struct DTensor {
  std::string name;
  int rows_in, cols_out, kind;   // 0 matrix (bf16 [out_pad][ld]), 1 bias, 2 gain (fp32)
  size_t off; int ld, rows_pad;
  int taps, cin, cin_pad;        // matrices: stored input index = tap*cin_pad + c for logical tap*cin + c
};
struct DTap { void* dst; size_t cap; };
inline size_t rup(size_t x, size_t a) { return (x + a - 1) / a * a; }
constexpr int GROUPS = 32;
}  // namespace

struct dec_ctx {
  dec_config cfg;
  int device = 0;
  hipStream_t stream = nullptr;
  std::vector<DTensor> tensors;
  std::unordered_map<std::string, int> index;
  size_t weight_bytes = 0;
  unsigned char* weights = nullptr;
  unsigned char* ws = nullptr;
  size_t ws_bytes = 0;
  mutable std::string err;
  std::map<std::string, DTap> taps;
  std::vector<int> host_map;
  hipEvent_t map_done = nullptr;
};

namespace {

dit_status dfail(const dec_ctx* c, dit_status st, const char* fmt, ...) {
  char buf[512];
  va_list ap; va_start(ap, fmt); vsnprintf(buf, sizeof buf, fmt, ap); va_end(ap);
  if (c) c->err = buf;
  return st;
}
#define DHIP(c, call)                                                                              \
  do {                                                                                             \
    hipError_t e_ = (call);                                                                        \
    if (e_ != hipSuccess) return dfail(c, DIT_EDEVICE, "%s: %s", #call, hipGetErrorString(e_));    \
  } while (0)

void add_vec(dec_ctx* c, const std::string& name, int n, int kind) {
  DTensor t;
  t.name = name; t.rows_in = 1; t.cols_out = n; t.kind = kind; t.off = c->weight_bytes;
  t.ld = t.rows_pad = t.taps = t.cin = t.cin_pad = 0;
  c->weight_bytes += rup((size_t)n * 4, 256);
  c->index[name] = (int)c->tensors.size();
  c->tensors.push_back(t);
}
void add_conv(dec_ctx* c, const std::string& name, int cin, int cout, int k) {
  DTensor t;
  t.name = name + ".w"; t.taps = k * k * (k == 3 && c->cfg.temporal ? 3 : 1); t.cin = cin; t.cin_pad = (int)rup(cin, 64);
  t.rows_in = t.taps * cin; t.cols_out = cout; t.kind = 0; t.off = c->weight_bytes;
  t.ld = t.taps * t.cin_pad; t.rows_pad = (int)rup(cout, 256);
  c->weight_bytes += rup((size_t)t.rows_pad * t.ld * 2, 256);
  c->index[t.name] = (int)c->tensors.size();
  c->tensors.push_back(t);
  add_vec(c, name + ".b", cout, 1);
}
void add_gn(dec_ctx* c, const std::string& name, int ch) { add_vec(c, name + ".g", ch, 2); add_vec(c, name + ".b", ch, 1); }
void add_res(dec_ctx* c, const std::string& name, int cin, int cout) {
  add_gn(c, name + ".gn1", cin); add_conv(c, name + ".conv1", cin, cout, 3);
  add_gn(c, name + ".gn2", cout); add_conv(c, name + ".conv2", cout, cout, 3);
  if (cin != cout) add_conv(c, name + ".short", cin, cout, 1);
}
const DTensor* find(const dec_ctx* c, const std::string& n) {
  auto it = c->index.find(n);
  return it == c->index.end() ? nullptr : &c->tensors[it->second];
}
const bf16_t* Wm(const dec_ctx* c, const std::string& n) { return (const bf16_t*)(c->weights + find(c, n)->off); }
const float* Wv(const dec_ctx* c, const std::string& n) { return (const float*)(c->weights + find(c, n)->off); }
int Wld(const dec_ctx* c, const std::string& n) { return find(c, n)->ld; }

uint64_t fnv(const std::string& s) {
  uint64_t h = 0xCBF29CE484222325ull;
  for (unsigned char ch : s) { h ^= ch; h *= 0x100000001B3ull; }
  return h;
}
uint64_t mix(uint64_t x) {
  uint64_t z = x + 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
uint16_t h_f2bf(float f) {
  uint32_t u; memcpy(&u, &f, 4);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

struct Layout {
  size_t map, xa, xb, t, img, act, q, k, v, vt, sc, pm, gnp, gst, out4, partial, total;
  int Hf, Wf, P0, P0pad;          // final image size; latent pixels and their padding to 64
  int n_out;                      // images at the output (a video's frame count grows with the frame rate)
};
constexpr size_t PARTIAL_BYTES = (size_t)256 * 128 * 128 * 4;

// latent sides 1..4096, h*w a multiple of 64 (whole k-slabs in the attention products) and at
// most 65536 (the score matrix is held whole); the final image at most 65535 rows, all output
// pixels together below 2^29 (product rows are 32-bit), and what one tile of a convolution
// reaches in its stack of bordered images (its own rows' windows plus the taps: an image, or three
// frames of a video) below 2^31 elements (32-bit byte offsets from the tile's first window);
// n images: 1..GN_MAX_BATCH, and with n > 1 h*w a multiple of 256 (group-norm chunks must not
// straddle images)
// frames (images) at the output of a video decoder that starts with n: 2F - 1 per frame-rate doubling
long long frames_out(const dec_ctx* c, long long n) {
  if (c->cfg.temporal)
    for (int l = 0; l < c->cfg.t_up; ++l) n = 2 * n - 1;
  return n;
}
bool size_ok(const dec_ctx* c, int n, int h, int w) {
  if (!(h >= 1 && w >= 1 && h <= 4096 && w <= 4096 && ((long long)h * w) % 64 == 0 && (long long)h * w <= 65536)) return false;
  const long long nf = n >= 1 ? frames_out(c, n) : 0;
  if (n < 1 || nf > GN_MAX_BATCH || (nf > 1 && ((long long)h * w) % 256 != 0)) return false;
  const int up = 1 << (c->cfg.n_levels - 1);
  const long long Hf = (long long)h * up, Wf = (long long)w * up;
  if (Hf > 65535 || nf * Hf * Wf >= (1LL << 31) / 4) return false;
  // the widest bordered image of each level: its own width, and the previous level's after the upsampling
  const long long reach = c->cfg.temporal ? 3 : 1;
  long long H = h, W = w, worst = 0;
  int prev = std::max(c->cfg.channels[0], 64);
  for (int l = 0; l < c->cfg.n_levels; ++l) {
    const int ch = c->cfg.channels[l];
    worst = std::max(worst, reach * (H + 2) * (W + 2) * std::max(ch, prev));
    prev = ch;
    if (l != c->cfg.n_levels - 1) { H *= 2; W *= 2; worst = std::max(worst, reach * (H + 2) * (W + 2) * ch); }
  }
  return worst < (1LL << 31);
}

void plan(const dec_ctx* c, int n, int h, int w, Layout& L) {
  const dec_config& g = c->cfg;
  const int up = 1 << (g.n_levels - 1);
  L.Hf = h * up; L.Wf = w * up;
  L.P0 = h * w; L.P0pad = (int)rup(L.P0, 256);        // rows of k as the product's second operand are read up to a multiple of 256
  // the largest stream / image / intermediate over the levels
  // (n streams / bordered images back to back; a video's frame count grows on the way and its stacks of
  // bordered images start with two zero frames)
  size_t max_x = 0, max_img = 0;
  int H = h, W = w;
  int prev = g.channels[0];
  size_t F = n;
  const size_t pad = g.temporal ? 2 : 0;
  max_x = std::max(max_x, F * H * W * prev);
  max_img = std::max(max_img, (F + pad) * (H + 2) * (W + 2) * std::max(prev, 64));
  for (int l = 0; l < g.n_levels; ++l) {
    const int ch = g.channels[l];
    max_x = std::max(max_x, F * H * W * std::max(ch, prev));
    max_img = std::max(max_img, (F + pad) * (H + 2) * (W + 2) * std::max(ch, prev));
    prev = ch;
    if (l != g.n_levels - 1) {
      if (g.temporal && l < g.t_up) F = 2 * F - 1;
      H *= 2; W *= 2;
      max_img = std::max(max_img, (F + pad) * (H + 2) * (W + 2) * ch);
      max_x = std::max(max_x, F * H * W * ch);
    }
  }
  L.n_out = (int)F;
  const size_t C0 = g.channels[0];
  size_t o = 0;
  auto take = [&](size_t bytes) { const size_t at = o; o += rup(bytes, 256); return at; };
  L.map = take((size_t)rup(L.P0, 64) * 4);
  L.xa = take(max_x * 4); L.xb = take(max_x * 4); L.t = take(max_x * 4);
  L.img = take(max_img * 2 + 4096);
  L.act = take(max_x * 2);                                    // bf16 copy of the stream (1x1 shortcuts, attention input)
  L.q = take((size_t)n * L.P0 * C0 * 2); L.k = take(((size_t)(n - 1) * L.P0 + L.P0pad) * C0 * 2); L.v = take((size_t)n * L.P0 * C0 * 2);
  L.vt = take(rup(C0, 256) * rup(L.P0, 64) * 2);            // read as a second operand: rows up to a multiple of 256
  L.sc = take((size_t)L.P0 * L.P0 * 4);
  L.pm = take((size_t)L.P0 * rup(L.P0, 64) * 2);
  // channel sums per chunk of 64 pixels at least (the smallest wave height of a product tile)
  L.gnp = take(std::max(group_norm_partial_bytes((long long)L.n_out * L.Hf * L.Wf, 1024), max_x / 64 * 8 + 2 * 1024 * 8));
  L.gst = take(GN_STATS_BYTES);
  L.out4 = take((size_t)L.n_out * L.Hf * L.Wf * 4 * 4);
  L.partial = take(PARTIAL_BYTES);
  L.total = o;
}

GemmProblem prob(const bf16_t* A, int lda, const bf16_t* W, int ldw, const float* bias, int M, int N, int K, int kind,
                 void* out, int ldc) {
  GemmProblem p;
  p.A = A; p.lda = lda; p.W = W; p.ldw = ldw; p.bias = bias; p.M = M; p.N = N; p.K = K;
  p.out_kind = kind; p.out = out; p.ldc = ldc; p.gate = nullptr; p.gate_stride = 0; p.row_req = nullptr;
  p.tiles_m = p.tiles_n = p.tile_start = 0;
  p.qk = QkNorm{};
  p.conv_w = 0; p.conv_cin = 0;
  return p;
}

struct Fwd {
  dec_ctx* c; const Layout& L; unsigned char* ws; hipStream_t s;
  mutable int B;                           // images (frames) at the current level
  int kt = 1;                              // frame taps of the 3x3 convolutions: 1, or 3 for a video
  // the buffer whose per-chunk channel sums the last convolution left in the group-norm scratch
  mutable const float* stats_of = nullptr;
  mutable int stats_chunks = 0;
  template <class T> T* at(size_t off) const { return (T*)(ws + off); }
  int gemm(std::initializer_list<GemmProblem> ps) const {
    GemmBatch b;
    b.n = 0; b.total_tiles = 0;
    for (const GemmProblem& p : ps) {
      if (p.out == stats_of) stats_of = nullptr;      // the buffer changes: its sums are stale
      b.p[b.n++] = p;
    }
    b.partial = at<float>(L.partial); b.partial_bytes = PARTIAL_BYTES;
    return launch_gemm(s, b);
  }
  // 3x3 convolution of the bordered bf16 image `img` (H x W, cin_pad channels) into fp32 rows
  // (a video's stack starts with two zero frames: `img` is the stack, frame() its first real image)
  void conv3(const std::string& name, const bf16_t* img, int H, int W, int kind, float* out, int ldc, bool sums = true) const {
    const DTensor* t = find(c, name + ".w");
    GemmProblem p = prob(img, t->cin_pad, Wm(c, name + ".w"), t->ld, Wv(c, name + ".b"), B * H * W, t->cols_out,
                         9 * kt * t->cin_pad, kind, out, ldc);
    p.conv_w = W; p.conv_cin = t->cin_pad; p.conv_img = H * W; p.conv_kt = kt;
    const bool want = sums && (kind == OUT_F32 || kind == OUT_RESID_F32);   // a group norm reads `out` next
    if (want) p.stats = at<float>(L.gnp);
    const int tile = gemm({p});
    if (want) {
      const int rows = gemm_stats_rows(tile);
      // chunks per image: one per wave row of a tile (a lone image may end inside a tile; with
      // several, H*W is a multiple of every chunk height)
      stats_of = out; stats_chunks = B == 1 ? (H * W + 2 * rows - 1) / (2 * rows) * 2 : H * W / rows;
    }
  }
  void gn(const std::string& name, const float* x, bf16_t* out, int H, int W, int C, int silu, int pad) const {
    launch_group_norm(s, x, Wv(c, name + ".g"), Wv(c, name + ".b"), out, at<float>(L.gnp), at<float2>(L.gst), H, W, C,
                      GROUPS, silu, pad, x == stats_of ? stats_chunks : 0, B);
  }
  // first real image of the stack of bordered images of H x W x C
  bf16_t* frame(int H, int W, int C) const { return at<bf16_t>(L.img) + (kt == 3 ? (size_t)2 * (H + 2) * (W + 2) * C : 0); }
  void zero_img(int H, int W, int C) const {       // the border must be zero; the interior is overwritten
    if (kt == 3) launch_fill_u16(s, at<bf16_t>(L.img), (long long)2 * (H + 2) * (W + 2) * C, 0);   // the two frames before the first
    launch_zero_border(s, frame(H, W, C), H, W, C, B);
  }
  // x (cin channels, in `x`) -> result (cout channels) in `y`; y == x when cin == cout
  void res(const std::string& name, float* x, float* y, int H, int W, int cin, int cout) const {
    bf16_t* img = at<bf16_t>(L.img);
    float* t = at<float>(L.t);
    zero_img(H, W, cin);
    gn(name + ".gn1", x, frame(H, W, cin), H, W, cin, 1, 1);
    conv3(name + ".conv1", img, H, W, OUT_F32, t, cout);
    if (cin != cout) {
      launch_cast_bf16(s, x, at<bf16_t>(L.act), (long long)B * H * W * cin);
      gemm({prob(at<bf16_t>(L.act), cin, Wm(c, name + ".short.w"), Wld(c, name + ".short.w"), Wv(c, name + ".short.b"),
                 B * H * W, cout, cin, OUT_F32, y, cout)});
    }
    zero_img(H, W, cout);
    gn(name + ".gn2", t, frame(H, W, cout), H, W, cout, 1, 1);
    conv3(name + ".conv2", img, H, W, OUT_RESID_F32, y, cout);
  }
};

dit_status tap(dec_ctx* c, const std::string& name, const void* src, size_t bytes) {
  auto it = c->taps.find(name);
  if (it == c->taps.end()) return DIT_OK;
  if (bytes > it->second.cap) return dfail(c, DIT_ENOMEM, "tap %s needs %zu bytes, buffer has %zu", name.c_str(), bytes, it->second.cap);
  DHIP(c, hipMemcpyAsync(it->second.dst, src, bytes, hipMemcpyDeviceToDevice, c->stream));
  return DIT_OK;
}
#define DTAP(name, src, bytes)                                            \
  do {                                                                    \
    if (!c->taps.empty()) {                                               \
      dit_status st_ = tap(c, name, src, bytes);                          \
      if (st_ != DIT_OK) return st_;                                      \
    }                                                                     \
  } while (0)

}  // namespace

extern "C" {

dit_status dec_create(const dec_config* cfg, int device, void* hip_stream, dec_ctx** out) {
  if (!out) return DIT_EINVAL;
  *out = nullptr;
  if (!cfg) return DIT_EINVAL;
  const dec_config& g = *cfg;
  if (g.latent_ch < 1 || g.latent_ch > 64 || g.out_ch < 1 || g.out_ch > 4) return DIT_ESHAPE;
  if (g.n_levels < 1 || g.n_levels > DEC_MAX_LEVELS || g.n_res < 1) return DIT_EINVAL;
  for (int l = 0; l < g.n_levels; ++l) {
    const int ch = g.channels[l];
    if (ch != 64 && ch != 128 && ch != 256 && ch != 512 && ch != 1024) return DIT_ESHAPE;
  }
  if (g.channels[0] % 128) return DIT_ESHAPE;      // the mid-block attention transposes v in 128-channel slices
  if ((g.temporal != 0 && g.temporal != 1) || g.t_up < 0 || g.t_up > g.n_levels - 1 || (!g.temporal && g.t_up)) return DIT_EINVAL;
  dec_ctx* c = new dec_ctx();
  c->cfg = g; c->device = device; c->stream = (hipStream_t)hip_stream;
  const int* ch = g.channels;
  add_conv(c, "conv_in", g.latent_ch, ch[0], 3);
  add_res(c, "mid.res0", ch[0], ch[0]);
  add_gn(c, "mid.attn.gn", ch[0]);
  for (const char* n : {"q", "k", "v", "proj"}) add_conv(c, std::string("mid.attn.") + n, ch[0], ch[0], 1);
  add_res(c, "mid.res1", ch[0], ch[0]);
  int prev = ch[0];
  for (int l = 0; l < g.n_levels; ++l) {
    for (int r = 0; r < g.n_res; ++r)
      add_res(c, "up" + std::to_string(l) + ".res" + std::to_string(r), r == 0 ? prev : ch[l], ch[l]);
    prev = ch[l];
    if (l != g.n_levels - 1) add_conv(c, "up" + std::to_string(l) + ".upconv", ch[l], ch[l], 3);
  }
  add_gn(c, "out.gn", ch[g.n_levels - 1]);
  add_conv(c, "conv_out", ch[g.n_levels - 1], g.out_ch, 3);
  *out = c;
  return DIT_OK;
}

void dec_destroy(dec_ctx* c) {
  if (!c) return;
  if (c->map_done) { (void)hipEventSynchronize(c->map_done); (void)hipEventDestroy(c->map_done); }
  delete c;
}
const char* dec_last_error(const dec_ctx* c) { return c ? c->err.c_str() : "null context"; }
size_t dec_weight_bytes(const dec_ctx* c) { return c ? c->weight_bytes : 0; }
size_t dec_workspace_bytes(const dec_ctx* c, int n, int h, int w) {
  if (!c || !size_ok(c, n, h, w)) return 0;
  Layout L;
  plan(c, n, h, w, L);
  return L.total;
}

dit_status dec_bind(dec_ctx* c, void* w, size_t wb, void* ws, size_t wsb) {
  if (!c) return DIT_EINVAL;
  if (!w || !ws) return dfail(c, DIT_EINVAL, "null buffer");
  if (((uintptr_t)w & 255) || ((uintptr_t)ws & 255)) return dfail(c, DIT_EINVAL, "buffers must be 256-byte aligned");
  if (wb < c->weight_bytes) return dfail(c, DIT_ENOMEM, "weight arena has %zu bytes, needs %zu", wb, c->weight_bytes);
  c->weights = (unsigned char*)w; c->ws = (unsigned char*)ws; c->ws_bytes = wsb;
  return DIT_OK;
}

dit_status dec_init_weights(dec_ctx* c, uint64_t seed, float std) {
  if (!c) return DIT_EINVAL;
  if (!c->weights) return dfail(c, DIT_EINVAL, "dec_bind has not been called");
  if (!(std >= 0.f) || !std::isfinite(std)) return dfail(c, DIT_EINVAL, "std must be finite and non-negative");
  DHIP(c, hipSetDevice(c->device));
  DHIP(c, hipMemsetAsync(c->weights, 0, c->weight_bytes, c->stream));
  for (const DTensor& t : c->tensors) {
    const uint64_t key = mix(seed ^ (fnv(t.name) * 0x9E3779B97F4A7C15ull));
    if (t.kind == 0) {
      // logical input index tap*cin + c lives at column tap*cin_pad + c: one launch per tap, the
      // generator's counter offset by the tap's first logical element
      for (int tp = 0; tp < t.taps; ++tp)
        launch_init_matrix(c->stream, (bf16_t*)(c->weights + t.off) + (size_t)tp * t.cin_pad, t.cols_out, t.cin, t.ld,
                           key + (uint64_t)tp * t.cin * t.cols_out, std);
    } else if (t.kind == 2) {
      launch_fill_f32(c->stream, (float*)(c->weights + t.off), t.cols_out, 1.0f);
    }
  }
  DHIP(c, hipGetLastError());
  return DIT_OK;
}

int dec_frames_out(const dec_ctx* c, int n) { return c && n >= 1 ? (int)std::min<long long>(frames_out(c, n), 0x7FFFFFFF) : 0; }

int dec_tensor_count(const dec_ctx* c) { return c ? (int)c->tensors.size() : 0; }
dit_status dec_tensor_info(const dec_ctx* c, int i, char* name, size_t len, int* rows_in, int* cols_out, int* kind) {
  if (!c || i < 0 || i >= (int)c->tensors.size()) return DIT_EINVAL;
  const DTensor& t = c->tensors[i];
  if (name && len) { strncpy(name, t.name.c_str(), len - 1); name[len - 1] = 0; }
  if (rows_in) *rows_in = t.rows_in;
  if (cols_out) *cols_out = t.cols_out;
  if (kind) *kind = t.kind;
  return DIT_OK;
}

dit_status dec_set_tensor(dec_ctx* c, const char* name, const float* src, size_t n) {
  if (!c || !name || !src) return DIT_EINVAL;
  if (!c->weights) return dfail(c, DIT_EINVAL, "dec_bind has not been called");
  const DTensor* t = find(c, name);
  if (!t) return dfail(c, DIT_ENOTFOUND, "no tensor named %s", name);
  if (n != (size_t)t->rows_in * t->cols_out) return dfail(c, DIT_ESHAPE, "%s has %d x %d elements", name, t->rows_in, t->cols_out);
  DHIP(c, hipSetDevice(c->device));
  DHIP(c, hipStreamSynchronize(c->stream));
  if (t->kind == 0) {
    std::vector<uint16_t> buf((size_t)t->rows_pad * t->ld, 0);
    for (int i = 0; i < t->rows_in; ++i) {
      const int ki = (i / t->cin) * t->cin_pad + i % t->cin;
      for (int o = 0; o < t->cols_out; ++o) buf[(size_t)o * t->ld + ki] = h_f2bf(src[(size_t)i * t->cols_out + o]);
    }
    DHIP(c, hipMemcpy(c->weights + t->off, buf.data(), buf.size() * 2, hipMemcpyHostToDevice));
  } else {
    DHIP(c, hipMemcpy(c->weights + t->off, src, n * 4, hipMemcpyHostToDevice));
  }
  return DIT_OK;
}

dit_status dec_get_tensor(dec_ctx* c, const char* name, float* dst, size_t n) {
  if (!c || !name || !dst) return DIT_EINVAL;
  if (!c->weights) return dfail(c, DIT_EINVAL, "dec_bind has not been called");
  const DTensor* t = find(c, name);
  if (!t) return dfail(c, DIT_ENOTFOUND, "no tensor named %s", name);
  if (n != (size_t)t->rows_in * t->cols_out) return dfail(c, DIT_ESHAPE, "%s has %d x %d elements", name, t->rows_in, t->cols_out);
  DHIP(c, hipSetDevice(c->device));
  DHIP(c, hipStreamSynchronize(c->stream));
  if (t->kind == 0) {
    std::vector<uint16_t> buf((size_t)t->cols_out * t->ld);
    DHIP(c, hipMemcpy(buf.data(), c->weights + t->off, buf.size() * 2, hipMemcpyDeviceToHost));
    for (int i = 0; i < t->rows_in; ++i) {
      const int ki = (i / t->cin) * t->cin_pad + i % t->cin;
      for (int o = 0; o < t->cols_out; ++o) {
        const uint32_t u = (uint32_t)buf[(size_t)o * t->ld + ki] << 16;
        memcpy(&dst[(size_t)i * t->cols_out + o], &u, 4);
      }
    }
  } else {
    DHIP(c, hipMemcpy(dst, c->weights + t->off, n * 4, hipMemcpyDeviceToHost));
  }
  return DIT_OK;
}

dit_status dec_set_tap(dec_ctx* c, const char* point, void* dst, size_t bytes) {
  if (!c || !point || !dst) return DIT_EINVAL;
  c->taps[point] = DTap{dst, bytes};
  return DIT_OK;
}
void dec_clear_taps(dec_ctx* c) { if (c) c->taps.clear(); }

dit_status dec_forward(dec_ctx* c, int n, int h, int w, const float* latent, float* image) {
  if (!c) return DIT_EINVAL;
  if (!c->weights || !c->ws) return dfail(c, DIT_EINVAL, "dec_bind has not been called");
  if (!latent || !image) return dfail(c, DIT_EINVAL, "null latent or image");
  if (!size_ok(c, n, h, w))
    return dfail(c, DIT_ESHAPE, "%d latent(s) of %d x %d: sides 1..4096, pixel count a multiple of 64 (256 for a batch or a video) and at most 65536, "
                 "1..%d images or output frames with fewer than 2^29 pixels together", n, h, w, GN_MAX_BATCH);
  const dec_config& g = c->cfg;
  DHIP(c, hipSetDevice(c->device));
  Layout L;
  plan(c, n, h, w, L);
  if (L.total > c->ws_bytes) return dfail(c, DIT_ENOMEM, "workspace has %zu bytes, this call needs %zu", c->ws_bytes, L.total);
  hipStream_t s = c->stream;
  Fwd F{c, L, c->ws, s, n};
  F.kt = g.temporal ? 3 : 1;
  const int pad_frames = g.temporal ? 2 : 0;
  // identity column map of the mid-block's value transpose
  if (c->map_done) DHIP(c, hipEventSynchronize(c->map_done));
  else DHIP(c, hipEventCreateWithFlags(&c->map_done, hipEventDisableTiming));
  const int P0 = L.P0, P0c = (int)rup(P0, 64);
  c->host_map.resize(P0c);
  for (int i = 0; i < P0c; ++i) c->host_map[i] = i < P0 ? i : -1;
  DHIP(c, hipMemcpyAsync(c->ws + L.map, c->host_map.data(), (size_t)P0c * 4, hipMemcpyHostToDevice, s));
  DHIP(c, hipEventRecord(c->map_done, s));

  const int C0 = g.channels[0];
  float* xa = F.at<float>(L.xa); float* xb = F.at<float>(L.xb);
  bf16_t* img = F.at<bf16_t>(L.img);
  int H = h, W = w;
  // conv_in: latents (channels-first fp32) -> bordered bf16 images with the channels padded to 64
  const DTensor* tin = find(c, "conv_in.w");
  launch_fill_u16(s, img, (long long)(n + pad_frames) * (H + 2) * (W + 2) * tin->cin_pad, 0);
  launch_latent_to_image(s, latent, F.frame(H, W, tin->cin_pad), g.latent_ch, H, W, tin->cin_pad, n, g.temporal ? n : 0);
  F.conv3("conv_in", img, H, W, OUT_F32, xa, C0);
  // mid block
  F.res("mid.res0", xa, xa, H, W, C0, C0);
  DTAP("mid.res0", xa, (size_t)n * P0 * C0 * 4);
  {
    bf16_t* hn = F.at<bf16_t>(L.act);
    bf16_t* q = F.at<bf16_t>(L.q); bf16_t* k = F.at<bf16_t>(L.k); bf16_t* v = F.at<bf16_t>(L.v);
    bf16_t* vt = F.at<bf16_t>(L.vt); float* sc = F.at<float>(L.sc); bf16_t* pm = F.at<bf16_t>(L.pm);
    const int M0 = n * P0;
    F.gn("mid.attn.gn", xa, hn, H, W, C0, 0, 0);
    F.gemm({prob(hn, C0, Wm(c, "mid.attn.q.w"), Wld(c, "mid.attn.q.w"), Wv(c, "mid.attn.q.b"), M0, C0, C0, OUT_BF16, q, C0),
            prob(hn, C0, Wm(c, "mid.attn.k.w"), Wld(c, "mid.attn.k.w"), Wv(c, "mid.attn.k.b"), M0, C0, C0, OUT_BF16, k, C0),
            prob(hn, C0, Wm(c, "mid.attn.v.w"), Wld(c, "mid.attn.v.w"), Wv(c, "mid.attn.v.b"), M0, C0, C0, OUT_BF16, v, C0)});
    // per image: scores = q k^T (k is the second operand as it stands: [keys][C], C contiguous;
    // the tile may read rows of the next image or of the padding: their columns are not stored),
    // softmax, o = P v with v^T [C][keys] from the value transpose in 128-channel slices; o goes
    // to hn, which is free after the three products
    for (int b = 0; b < n; ++b) {
      const size_t ro = (size_t)b * P0 * C0;
      F.gemm({prob(q + ro, C0, k + ro, C0, nullptr, P0, P0, C0, OUT_F32, sc, P0)});
      launch_softmax_rows(s, sc, P0, pm, P0c, P0, P0, 1.4426950408889634f / sqrtf((float)C0));
      launch_v_transpose(s, v + ro, C0, 0, C0 / 128, 128, F.at<int>(L.map), P0c, vt, P0c);
      F.gemm({prob(pm, P0c, vt, P0c, nullptr, P0, C0, P0c, OUT_BF16, hn + ro, C0)});
    }
    F.gemm({prob(hn, C0, Wm(c, "mid.attn.proj.w"), Wld(c, "mid.attn.proj.w"), Wv(c, "mid.attn.proj.b"), M0, C0, C0,
                 OUT_RESID_F32, xa, C0)});
  }
  DTAP("mid.attn", xa, (size_t)n * P0 * C0 * 4);
  F.res("mid.res1", xa, xa, H, W, C0, C0);
  // up levels
  float* x = xa; float* other = xb;
  int prev = C0;
  for (int l = 0; l < g.n_levels; ++l) {
    const int ch = g.channels[l];
    for (int r = 0; r < g.n_res; ++r) {
      const std::string name = "up" + std::to_string(l) + ".res" + std::to_string(r);
      const int cin = r == 0 ? prev : ch;
      if (cin != ch) { F.res(name, x, other, H, W, cin, ch); std::swap(x, other); }
      else F.res(name, x, x, H, W, ch, ch);
    }
    prev = ch;
    DTAP("up" + std::to_string(l), x, (size_t)F.B * H * W * ch * 4);
    if (l != g.n_levels - 1) {
      const int frame_up = g.temporal && l < g.t_up;       // F frames -> 2F - 1: the first once, the others twice
      if (frame_up) F.B = 2 * F.B - 1;
      F.zero_img(2 * H, 2 * W, ch);
      launch_upsample_pad(s, x, F.frame(2 * H, 2 * W, ch), H, W, ch, F.B, frame_up);
      H *= 2; W *= 2;
      F.conv3("up" + std::to_string(l) + ".upconv", img, H, W, OUT_F32, other, ch);
      std::swap(x, other);
    }
  }
  // output: GN + SiLU + conv to out_ch channels
  F.zero_img(H, W, prev);
  F.gn("out.gn", x, F.frame(H, W, prev), H, W, prev, 1, 1);
  {
    const DTensor* to = find(c, "conv_out.w");
    // 27 taps: the 9-tap kernel once per frame tap kf, on the stack shifted by kf frames, adding up in that order
    bool direct = true;
    for (int kf = 0; kf < F.kt && direct; ++kf)
      direct = launch_conv3_small(s, img + (size_t)kf * (H + 2) * (W + 2) * to->cin_pad, Wm(c, "conv_out.w") + (size_t)kf * 9 * to->cin_pad,
                                  to->ld, kf == 0 ? Wv(c, "conv_out.b") : nullptr, image, H, W, to->cin_pad, g.out_ch, F.B, kf > 0);
    if (!direct) {
      F.conv3("conv_out", img, H, W, OUT_F32, F.at<float>(L.out4), 4, false);     // as a product, rows 4 wide, then compacted
      launch_compact_rows(s, F.at<float>(L.out4), 4, image, (long long)F.B * H * W, g.out_ch);
    }
  }
  DHIP(c, hipGetLastError());
  return DIT_OK;
}

}  // extern "C"
