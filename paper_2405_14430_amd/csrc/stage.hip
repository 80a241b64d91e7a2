// Stage runtime and C boundary (include/pfstage.h): configuration checks, carving of the caller's K/V buffer
// and workspace, and the per-layer launch sequence of one PipeFusion stage pass (Sec. 3.3) for the four block
// kinds.  Host code only; every arithmetic step runs in the kernels of the other files.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/pfstage.h"
#include "ops.h"

using namespace pf;

namespace {

thread_local std::string g_create_error;


inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Derived {
  int n, T, Tj, Lkv, Lp, Tp, Rmax, mod_chunks, n_streams;
  bool rope;      // q and k of the image rows are rotated (kind 3, or kind 2 with joint_rope)
  int B;          // images per call (classifier-free guidance runs the conditional and unconditional image together)
  size_t esz;
};

bool is_joint(int kind) { return kind == PF_BLOCK_MMDIT_JOINT || kind == PF_BLOCK_SINGLE_STREAM; }

const char *check_config(const pf_config *c, pf_status *st) {
  *st = PF_ERR_CONFIG;
  if (c->dtype != PF_F32 && c->dtype != PF_BF16) { *st = PF_ERR_DTYPE; return "unknown dtype"; }
  if (c->kind < 0 || c->kind > 3) return "unknown block kind";
  if (c->kernel_path != PF_PATH_AUTO && c->kernel_path != PF_PATH_SIMT) return "unknown kernel_path";
  if (c->n_layers < 1) return "n_layers must be >= 1";
  if (c->hidden < 8 || c->n_heads < 1 || c->head_dim < 8) return "hidden/n_heads/head_dim too small";
  if (c->hidden != c->n_heads * c->head_dim) return "hidden != n_heads * head_dim";
  if (c->head_dim % 8 || c->head_dim > 128) return "head_dim must be a multiple of 8 and <= 128";
  if (c->hidden > 8192) return "hidden must be <= 8192";
  if (c->mlp_dim < 8 || c->mlp_dim % 8) return "mlp_dim must be a positive multiple of 8";
  if (c->seq_img < 1 || c->n_patches < 1 || c->seq_img % c->n_patches) return "n_patches must divide seq_img";
  if (c->grid_h < 1 || c->grid_w < 1 || (int64_t)c->grid_h * c->grid_w != c->seq_img) return "grid_h * grid_w != seq_img";
  if (c->text_len < 0) return "text_len < 0";
  if (c->kind == PF_BLOCK_ADALN_SINGLE_XATTN) {
    if (c->text_len < 1) return "kind 1 needs text_len >= 1";
    if (c->cross_dim < 8 || c->cross_dim % 8) return "cross_dim must be a positive multiple of 8";
  }
  if (c->kind == PF_BLOCK_ADALN_ZERO && c->text_len != 0) return "kind 0 has no text";
  if (c->batch < 0 || c->batch > PF_MAX_BATCH) return "batch must be in [0, PF_MAX_BATCH] (0 means 1)";
  if (!(c->ln_eps > 0.f)) return "ln_eps must be > 0";
  if (c->joint_rope != 0 && c->joint_rope != 1) return "joint_rope must be 0 or 1";
  if (c->joint_rope && c->kind != PF_BLOCK_MMDIT_JOINT) return "joint_rope applies to kind 2 only (kind 3 always rotates)";
  if (c->txt_pre_only_last != 0 && c->txt_pre_only_last != 1) return "txt_pre_only_last must be 0 or 1";
  if (c->txt_pre_only_last && c->kind != PF_BLOCK_MMDIT_JOINT) return "txt_pre_only_last applies to kind 2 only";
  const bool rope = c->kind == PF_BLOCK_SINGLE_STREAM || c->joint_rope;
  if (rope && !(c->rope_theta > 1.f)) return "rope_theta must be > 1";
  if (rope && c->head_dim % 4) return "RoPE needs head_dim to be a multiple of 4";
  if (c->qk_norm != 0 && c->qk_norm != 1) return "qk_norm must be 0 or 1";
  if (c->qk_norm && (c->head_dim & (c->head_dim - 1))) return "qk_norm needs a power-of-two head_dim";
  *st = PF_OK;
  return nullptr;
}

Derived derive(const pf_config *c) {
  Derived d;
  d.n = c->seq_img / c->n_patches;
  d.T = c->text_len;
  d.Tj = is_joint(c->kind) ? c->text_len : 0;
  d.Lkv = c->seq_img + d.Tj;
  d.Lp = (int)align_up(d.Lkv, 128);
  d.Tp = (int)align_up(d.T > 0 ? d.T : 1, 128);
  d.Rmax = d.Lkv > d.T ? d.Lkv : d.T;   // rows of the largest pass (warm-up) and of the kind-1 text projection
  d.mod_chunks = c->kind == PF_BLOCK_SINGLE_STREAM ? 3 : 6;
  d.n_streams = c->kind == PF_BLOCK_MMDIT_JOINT ? 2 : 1;
  d.esz = dt_size(c->dtype);
  d.B = c->batch > 1 ? c->batch : 1;
  d.rope = c->kind == PF_BLOCK_SINGLE_STREAM || c->joint_rope;
  return d;
}

int use_path(const pf_config *c) { return (c->dtype == PF_BF16 && c->kernel_path == PF_PATH_AUTO) ? PATH_AUTO : PATH_SIMT; }

// Split of the key range of an attention launch.  The chip holds 512 attention workgroups of 128 queries at a time (two
// per CU; 256 of the 256-query kind), so a launch runs in ceil(workgroups / 512) rounds; the split count is picked to minimise a small cost model in units of
// one key tile: rounds x (tiles per split + fixed per-workgroup cost), a penalty for a first round that leaves CUs with
// a single workgroup (no second wave per SIMD to overlap with), and the combine pass that grows with the split count.
// Measured on MI355X: Flux-scale patch (384 blocks) 4 splits 478 us vs 2 splits 503 us vs none 583 us; SD3-scale patch
// (96 blocks) 5 splits 34 us vs 6 splits 38 us.
int choose_splits(int path, int nq, int H, int kv_rows, int head_dim) {
  const bool gen2 = path != PATH_SIMT && pf::g_attn_variant == 0 && (head_dim == 64 || head_dim == 72 || head_dim == 128);
  const int qtile = path == PATH_SIMT ? 64 : (gen2 ? attn_mfma2_qtile(nq) : 128);
  const int resident = qtile == 256 ? 256 : 512;   // workgroups the chip holds at a time
  const int ktile = path == PATH_SIMT ? 32 : 64;
  const int64_t blocks = (int64_t)((nq + qtile - 1) / qtile) * H;
  const int tiles = (kv_rows + ktile - 1) / ktile;
  int cap = tiles / 4;  // at least four tiles per split
  if (cap > 16) cap = 16;
  if (g_force_splits > 0) return g_force_splits < (cap < 1 ? 1 : cap) ? g_force_splits : (cap < 1 ? 1 : cap);
  int best = 1;
  double best_cost = 1e300;
  for (int sp = 1; sp <= (cap < 1 ? 1 : cap); ++sp) {
    const int64_t wgs = blocks * sp;
    const int64_t rounds = (wgs + resident - 1) / resident;
    const double fill = wgs >= resident ? 1.0 : (double)wgs / resident;
    double cost = (double)rounds * ((tiles + sp - 1) / sp + 4) * (1.0 + 0.5 * (1.0 - fill));
    if (sp > 1) cost += 2.0 + 0.5 * sp;
    if (cost < best_cost - 1e-9) { best_cost = cost; best = sp; }
  }
  return best;
}

size_t kv_layer_bytes(const pf_config *c, const Derived &d) {
  size_t self = 2 * (size_t)c->n_heads * d.Lp * c->head_dim * d.esz;
  size_t cross = c->kind == PF_BLOCK_ADALN_SINGLE_XATTN ? 2 * (size_t)c->n_heads * d.Tp * c->head_dim * d.esz : 0;
  return (self + cross) * d.B;
}

struct WsLayout {
  size_t mod, xres, h, qkv, a, u, xb, qc, rope, attn, total;
  size_t attn_bytes;
  int64_t lda_a;  // row stride of the attention-output buffer (d, or d+F for kind 3)
};

WsLayout ws_layout(const pf_config *c, const Derived &d) {
  WsLayout w{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  const size_t R = (size_t)d.Rmax * d.B, D = c->hidden, F = c->mlp_dim, e = d.esz;
  w.mod = take((size_t)d.B * d.n_streams * c->n_layers * d.mod_chunks * D * sizeof(float));
  w.xres = take(R * D * sizeof(float));
  w.h = take(R * D * e);
  w.qkv = take(R * 3 * D * e);
  if (c->kind == PF_BLOCK_SINGLE_STREAM) {
    w.lda_a = D + F;
    w.a = take(R * (D + F) * e);
    w.u = w.a;
  } else {
    w.lda_a = D;
    w.a = take(R * D * e);
    w.u = take(R * F * e);
  }
  if (c->kind == PF_BLOCK_ADALN_SINGLE_XATTN) {
    w.xb = take(R * D * e);
    w.qc = take(R * D * e);
  }
  if (d.rope) w.rope = take((size_t)d.Rmax * (size_t)(c->head_dim / 2) * 2 * sizeof(float));
  const int path = use_path(c);
  size_t ab = 0;
  // every query-row count a call can have: image-only patch, patch with the joint text rows, warm-up pass
  // (per image; with a batch the text rows of the MMDiT kind are a launch of their own)
  int shapes[5] = {d.n, d.n + d.Tj, d.Lkv, d.Tj > 0 ? d.Tj : d.n, c->seq_img};
  const int HB = c->n_heads * d.B;
  for (int nq : shapes) {
    size_t b = attention_ws_bytes(nq, HB, c->head_dim, choose_splits(path, nq, HB, d.Lkv, c->head_dim));
    if (b > ab) ab = b;
    if (c->kind == PF_BLOCK_ADALN_SINGLE_XATTN) {
      b = attention_ws_bytes(nq, HB, c->head_dim, choose_splits(path, nq, HB, d.T, c->head_dim));
      if (b > ab) ab = b;
    }
  }
  w.attn_bytes = ab;
  w.attn = take(ab);
  w.total = off;
  return w;
}

}  // namespace

struct pf_stage {
  pf_config cfg;
  Derived d;
  WsLayout w;
  std::vector<pf_layer_weights> img, txt;
  char *kv;
  char *ws;
  hipStream_t stream;
  bool ready = false;
  bool mod_valid[2] = {false, false};   // per stream: the modulation vectors in the workspace belong to the last cond
  std::string err;
  // profiling
  bool prof = false;
  // A mark is an event recorded on the stream; a launch of class cls spans the mark before it and its own mark
  // (cls < 0: start of a chain of launches).  Consecutive launches share the mark between them, so profiling adds one
  // event per launch, not two.
  struct Mark { int cls; hipEvent_t ev; };
  std::vector<Mark> events;
  std::vector<hipEvent_t> pool;
  bool chain_open = false;

  // Layer l of the caller's K/V buffer: [K of image 0 .. B-1][V^T of image 0 .. B-1][cross K ...][cross V^T ...], each
  // image's part head-major.  img_elems / ximg_elems: elements between consecutive images.
  size_t img_elems() const { return (size_t)cfg.n_heads * d.Lp * cfg.head_dim; }
  size_t ximg_elems() const { return (size_t)cfg.n_heads * d.Tp * cfg.head_dim; }
  char *kptr(int l) const { return kv + (size_t)l * kv_layer_bytes(&cfg, d); }
  char *vptr(int l) const { return kptr(l) + d.B * img_elems() * d.esz; }
  char *kcptr(int l) const { return kptr(l) + 2 * d.B * img_elems() * d.esz; }
  char *vcptr(int l) const { return kcptr(l) + d.B * ximg_elems() * d.esz; }
  // modulation vectors: [image][stream][layer][chunks * hidden]
  size_t mod_img_stride() const { return (size_t)d.n_streams * cfg.n_layers * d.mod_chunks * cfg.hidden; }
  float *mod(int stream_idx, int l, int b = 0) const {
    return (float *)(ws + w.mod) + b * mod_img_stride() + ((size_t)stream_idx * cfg.n_layers + l) * d.mod_chunks * cfg.hidden;
  }
};

namespace {

pf_status fail(pf_stage *s, pf_status st, const std::string &msg) {
  if (s) s->err = msg; else g_create_error = msg;
  return st;
}

hipEvent_t get_event(pf_stage *s) {
  if (!s->pool.empty()) { hipEvent_t e = s->pool.back(); s->pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  (void)hipEventCreate(&e);
  return e;
}

// Runs one launch, optionally bracketed by an event pair for the per-class timing.
template <typename Fn>
hipError_t run(pf_stage *s, int cls, Fn &&fn) {
  if (!s->prof) return fn();
  if (!s->chain_open) {
    pf_stage::Mark m{-1, get_event(s)};
    (void)hipEventRecord(m.ev, s->stream);
    s->events.push_back(m);
    s->chain_open = true;
  }
  hipError_t e = fn();
  pf_stage::Mark m{cls, get_event(s)};
  (void)hipEventRecord(m.ev, s->stream);
  s->events.push_back(m);
  return e;
}

#define PF_TRY(expr)                                                                       \
  do {                                                                                     \
    hipError_t e__ = (expr);                                                               \
    if (e__ != hipSuccess)                                                                 \
      return fail(s, PF_ERR_DEVICE, std::string(#expr) + ": " + hipGetErrorString(e__));   \
  } while (0)

hipError_t gemm(pf_stage *s, int cls, const void *A, int64_t lda, const void *W, int64_t ldw, const void *bias,
                void *C, int64_t ldc, int M, int N, int K, int epilogue, int gelu_from, const float *gate,
                const float *R, int64_t ldr, void *C2, int64_t ldc2, const GemmArgsKv *kvr = nullptr, int gate_seg = 0) {
  GemmArgs g{};
  if (kvr) g.kvr = *kvr;
  if (gate && gate_seg > 0 && s->d.B > 1) { g.gate_seg = gate_seg; g.gate_stride = (int64_t)s->mod_img_stride(); }
  g.dt = s->cfg.dtype; g.path = use_path(&s->cfg);
  g.A = A; g.lda = lda; g.W = W; g.ldw = ldw; g.bias = bias; g.C = C; g.ldc = ldc; g.M = M; g.N = N; g.K = K;
  g.epilogue = epilogue; g.gelu_from = gelu_from; g.gelu_tanh = s->cfg.gelu_tanh; g.gate = gate; g.R = R; g.ldr = ldr;
  g.C2 = C2; g.ldc2 = ldc2;
  return run(s, cls, [&] { return launch_gemm(g, s->stream); });
}

// (nq = query rows per image; every launch covers all images of the call)
// Split count of an attention launch of this stage: the occupancy heuristic, lowered if needed so that the partial
// results never exceed the workspace region reserved for them.
int plan_splits(const pf_stage *s, int nq, int kv_rows) {
  const int path = use_path(&s->cfg);
  const int HB = s->cfg.n_heads * s->d.B;
  int splits = choose_splits(path, nq, HB, kv_rows, s->cfg.head_dim);
  while (splits > 1 && attention_ws_bytes(nq, HB, s->cfg.head_dim, splits) > s->w.attn_bytes) --splits;
  return splits;
}

hipError_t attention(pf_stage *s, int cls, const void *q, int64_t ldq, const void *kb, const void *vb, int kv_rows,
                     int rows_padded, void *out, int64_t ldo, int nq, bool q_prescaled = false) {
  AttnArgs a{};
  a.dt = s->cfg.dtype; a.path = use_path(&s->cfg);
  a.q = q; a.ldq = ldq; a.kbuf = kb; a.vtbuf = vb; a.kv_rows = kv_rows; a.rows_padded = rows_padded;
  a.n_heads = s->cfg.n_heads; a.head_dim = s->cfg.head_dim; a.out = out; a.ldo = ldo; a.nq = nq;
  a.batch = s->d.B;
  a.q_prescaled = q_prescaled ? 1 : 0;
  a.splits = plan_splits(s, nq, kv_rows);
  a.ws = (float *)(s->ws + s->w.attn);
  hipError_t e = run(s, cls, [&] { return a.path == PATH_SIMT ? launch_attn_simt(a, s->stream) : launch_attn_bf16(a, s->stream); });
  if (e != hipSuccess) return e;
  if (a.splits > 1) e = run(s, PF_KC_ATTN_COMBINE, [&] { return launch_attn_combine(a, s->stream); });
  return e;
}

// QKV projection of `rows` rows plus the write of their K/V into the layer's buffers.  Rows are image-major, `seg` per
// image (rows = B * seg); inside an image, row r goes to buffer row (r < split ? row0a + r : row0b + r - split).  When
// the bf16 GEMM's vectorised epilogue can do it, k and v go straight from the accumulators into K / V^T (q, and RoPE
// through `rope_tab`, likewise); otherwise the projection lands in the qkv workspace and the scatter kernel moves (and
// rotates) it, one launch per image and row range.
// How the QKV projection of a stream reaches the buffers: through the GEMM epilogue, or through the scatter kernel,
// which rewrites q in fp32 only when it normalises or rotates.
enum { ROUTE_FUSED = 0, ROUTE_SCATTER_REWRITE, ROUTE_SCATTER_PLAIN };
int qkv_route(const pf_stage *s, const void *hs, const pf_layer_weights &lw, const char *qs, bool rope) {
  const pf_config &c = s->cfg;
  const int D = c.hidden;
  GemmArgs probe{};
  probe.dt = c.dtype; probe.path = use_path(&c); probe.A = hs; probe.lda = D; probe.W = lw.w_qkv; probe.ldw = D;
  probe.bias = lw.b_qkv; probe.C = (void *)qs; probe.ldc = 3 * D; probe.M = 1; probe.N = 3 * D; probe.K = D; probe.epilogue = 0;
  probe.gelu_from = 3 * D;
  probe.kvr = GemmArgsKv{(void *)qs, (void *)qs, s->d.Lp, c.head_dim, D, 0, 0, 0, nullptr, 0, 0, 0.f};
  if (g_fuse_kv_route && !c.qk_norm && gemm_kv_route_supported(probe)) return ROUTE_FUSED;   // the fused route has no q / k RMSNorm
  return (rope || c.qk_norm) ? ROUTE_SCATTER_REWRITE : ROUTE_SCATTER_PLAIN;
}

// q_scale != 0: q is to leave this function multiplied by it (folded into whichever fp32 step writes q; the caller only
// asks for it when every q row of the coming attention launch goes through such a step).
pf_status qkv_project(pf_stage *s, const void *hs, const pf_layer_weights &lw, char *qs, int seg, char *kb, char *vb,
                      int split, int row0a, int row0b, const void *rope_tab, int tok0, bool rope, float q_scale) {
  const pf_config &c = s->cfg;
  const Derived &d = s->d;
  const int D = c.hidden;
  const int rows = seg * d.B;
  GemmArgsKv kvr{kb, vb, d.Lp, c.head_dim, D, split, row0a, row0b, rope ? rope_tab : nullptr, d.B > 1 ? seg : 0,
                 (int64_t)s->img_elems(), q_scale};
  if (qkv_route(s, hs, lw, qs, rope) == ROUTE_FUSED) {
    PF_TRY(gemm(s, PF_KC_GEMM_QKV, hs, D, lw.w_qkv, D, lw.b_qkv, qs, 3 * D, rows, 3 * D, D, 0, 3 * D, nullptr, nullptr, 0,
                nullptr, 0, &kvr));
    return PF_OK;
  }
  PF_TRY(gemm(s, PF_KC_GEMM_QKV, hs, D, lw.w_qkv, D, lw.b_qkv, qs, 3 * D, rows, 3 * D, D, 0, 3 * D, nullptr, nullptr, 0,
              nullptr, 0));
  hipStream_t st = s->stream;
  for (int b = 0; b < d.B; ++b) {
    char *qb = qs + (size_t)b * seg * 3 * D * d.esz;
    char *kbb = kb + (size_t)b * s->img_elems() * d.esz, *vbb = vb + (size_t)b * s->img_elems() * d.esz;
    if (split > 0) {
      ScatterArgs sa{c.dtype, qb, 3 * D, kbb, vbb, d.Lp, c.n_heads, c.head_dim, row0a, split, rope ? 1 : 0, -1, c.grid_w, c.rope_theta};
      if (c.qk_norm) { sa.q_norm_w = lw.q_norm_w; sa.k_norm_w = lw.k_norm_w; sa.norm_eps = c.ln_eps; }
      sa.q_scale = q_scale;
      PF_TRY(run(s, PF_KC_KV_SCATTER, [&] { return launch_kv_scatter(sa, st); }));
    }
    ScatterArgs sb{c.dtype, qb + (size_t)split * 3 * D * d.esz, 3 * D, kbb, vbb, d.Lp, c.n_heads, c.head_dim, row0b, seg - split,
                   rope ? 1 : 0, tok0, c.grid_w, c.rope_theta};
    if (c.qk_norm) { sb.q_norm_w = lw.q_norm_w; sb.k_norm_w = lw.k_norm_w; sb.norm_eps = c.ln_eps; }
    sb.q_scale = q_scale;
    PF_TRY(run(s, PF_KC_KV_SCATTER, [&] { return launch_kv_scatter(sb, st); }));
  }
  return PF_OK;
}

// Device-to-device copy of B blocks of `block` floats each, source blocks src_pitch floats apart, destination blocks
// dst_pitch floats apart (one plain copy when both are dense or B = 1).
hipError_t copy_blocks(float *dst, size_t dst_pitch, const float *src, size_t src_pitch, size_t block, int B, hipStream_t st) {
  if (B == 1 || (dst_pitch == block && src_pitch == block))
    return hipMemcpyAsync(dst, src, (size_t)B * block * sizeof(float), hipMemcpyDeviceToDevice, st);
  return hipMemcpy2DAsync(dst, dst_pitch * sizeof(float), src, src_pitch * sizeof(float), block * sizeof(float), B,
                          hipMemcpyDeviceToDevice, st);
}

// The block stack on image rows [img_off, img_off + n_img) of each of the B images of the call and, for the joint kinds,
// on the T text rows of each image when `text` is given.  x_img / y_img: [B][n_img][D]; cond: [B][D or 6D]; text /
// text_out: [B][T][D].  Residual rows live in the workspace when text rows ride along: per image [text; image] for the
// single-stream kind (one weight set for both), all text rows then all image rows for the MMDiT kind (one weight set
// per stream, so each stream is one contiguous GEMM operand).
pf_status forward(pf_stage *s, const float *x_img, int n_img, int img_off, const float *cond, const float *text,
                  float *y_img, float *text_out, bool same_cond = false) {
  const pf_config &c = s->cfg;
  const Derived &d = s->d;
  const WsLayout &w = s->w;
  const int D = c.hidden, F = c.mlp_dim, dt = c.dtype, B = d.B;
  const size_t e = d.esz;
  const int Tt = (text && d.Tj) ? d.Tj : 0;   // text rows per image processed by this call
  const int R = Tt + n_img;                   // rows per image
  const bool single = c.kind == PF_BLOCK_SINGLE_STREAM;
  const size_t mstride = s->mod_img_stride();
  hipStream_t st = s->stream;
  char *ws = s->ws;
  float *xres = (float *)(ws + w.xres);
  char *h = ws + w.h, *qkv = ws + w.qkv, *a = ws + w.a, *u = ws + w.u;

  // Residual rows.  With text rows riding along they are gathered in the workspace.  Without, nothing is copied: the
  // first layer reads x_img directly, the first residual GEMM writes into the output buffer (or the workspace when
  // the caller wants no output) and everything after that runs in place there.
  float *xbuf = xres;          // where updated residual rows live
  const float *xsrc = xres;    // where the current residual rows are read from (x_img until the first update)
  // text block / image block of the residual rows: first row and distance between images, in rows
  const size_t t_row0 = 0, i_row0 = single ? (size_t)Tt : (size_t)B * Tt;
  const size_t t_pitch = single ? (size_t)R : (size_t)Tt, i_pitch = single ? (size_t)R : (size_t)n_img;
  if (Tt) {
    PF_TRY(run(s, PF_KC_COPY, [&] { return copy_blocks(xres + t_row0 * D, t_pitch * D, text, (size_t)Tt * D, (size_t)Tt * D, B, st); }));
    PF_TRY(run(s, PF_KC_COPY, [&] { return copy_blocks(xres + i_row0 * D, i_pitch * D, x_img, (size_t)n_img * D, (size_t)n_img * D, B, st); }));
  } else {
    xsrc = x_img;
    if (y_img) xbuf = y_img;
  }

  // a0: modulation vectors of every layer, stream and image, one launch per 16 of them
  {
    ModBatch mb{};
    const int out_dim = d.mod_chunks * D;
    const int table = c.kind == PF_BLOCK_ADALN_SINGLE_XATTN;
    const size_t cdim = table ? (size_t)6 * D : (size_t)D;
    auto flush = [&](int od) -> hipError_t {
      if (mb.count == 0) return hipSuccess;
      hipError_t e2 = run(s, PF_KC_MODULATION, [&] { return launch_modulation_batch(dt, mb, od, D, table, st); });
      mb.count = 0;
      return e2;
    };
    // streams whose vectors must be derived in this call: all that run, unless the caller vouches for the cond
    bool need[2] = {false, false};
    for (int si = 0; si < d.n_streams; ++si) {
      const bool runs = !(c.kind == PF_BLOCK_MMDIT_JOINT && si == 0 && !Tt);   // text stream idle without text rows
      need[si] = runs && !(same_cond && s->mod_valid[si]);
      if (!same_cond) s->mod_valid[si] = false;
      if (need[si] && !cond) return fail(s, PF_ERR_NULL, "cond is NULL but modulation vectors have to be derived");
    }
    for (int b = 0; b < B; ++b)
      for (int l = 0; l < c.n_layers; ++l)
        for (int si = 0; si < d.n_streams; ++si) {
          if (!need[si]) continue;
          const pf_layer_weights &lw = (d.n_streams == 2 && si == 0) ? s->txt[l] : s->img[l];
          mb.w[mb.count] = lw.w_mod; mb.b[mb.count] = lw.b_mod; mb.c[mb.count] = cond + b * cdim;
          mb.out[mb.count] = s->mod(si, l, b);
          if (c.txt_pre_only_last && si == 0 && l == c.n_layers - 1 && d.n_streams == 2) {
            // two chunks (shift, scale) instead of six: a launch of its own, the batch shares one output width
            ModBatch one{};
            one.w[0] = mb.w[mb.count]; one.b[0] = mb.b[mb.count]; one.c[0] = mb.c[mb.count]; one.out[0] = mb.out[mb.count];
            one.count = 1;
            PF_TRY(run(s, PF_KC_MODULATION, [&] { return launch_modulation_batch(dt, one, 2 * D, D, table, st); }));
            continue;
          }
          if (++mb.count == ModBatch::kMax) PF_TRY(flush(out_dim));
        }
    PF_TRY(flush(out_dim));
    for (int si = 0; si < d.n_streams; ++si)
      if (need[si]) s->mod_valid[si] = true;
  }

  const int row0_img = d.Tj + img_off;   // buffer row of the first image row of this call
  // The bf16 attention kernel has a variant that takes q already multiplied by log2(e) / sqrt(dh); the factor is folded
  // into the fp32 step that writes q (GEMM epilogue, or the scatter kernel when it normalises / rotates).
  const bool pre_ok = use_path(&c) == PATH_AUTO && pf::g_attn_variant == 0 && attn_mfma2_takes_prescaled_q(c.head_dim) &&
                      g_fold_q_scale;
  const float q_fold = 1.4426950408889634f / sqrtf((float)c.head_dim);
  bool q_pre = false;
  // (cos, sin) of the RoPE angles of one image's rows, shared by all layers and images of the call: [text; image] rows
  // for the single-stream kind, the image rows alone for the two-stream kind (its text stream is not rotated)
  if (single)
    PF_TRY(run(s, PF_KC_KV_SCATTER, [&] { return launch_rope_table(ws + w.rope, R, Tt, img_off, c.grid_w, c.head_dim, c.rope_theta, st); }));
  else if (d.rope)
    PF_TRY(run(s, PF_KC_KV_SCATTER, [&] { return launch_rope_table(ws + w.rope, n_img, 0, img_off, c.grid_w, c.head_dim, c.rope_theta, st); }));
  for (int l = 0; l < c.n_layers; ++l) {
    char *kb = s->kptr(l), *vb = s->vptr(l);
    if (single) {
      const pf_layer_weights &lw = s->img[l];
      const float *m = s->mod(0, l);
      const int RT = B * R;
      PF_TRY(run(s, PF_KC_LN_MODULATE, [&] { return launch_ln_modulate(dt, xsrc, D, m, m + D, c.ln_eps, h, D, RT, D, 1, st, B > 1 ? R : 0, mstride); }));
      {
        const bool pre = pre_ok && qkv_route(s, h, lw, qkv, true) != ROUTE_SCATTER_PLAIN;
        pf_status qs_ = qkv_project(s, h, lw, qkv, R, kb, vb, Tt, 0, row0_img, ws + w.rope, img_off, true, pre ? q_fold : 0.f);
        if (qs_ != PF_OK) return qs_;
        q_pre = pre;
      }
      // MLP branch runs in parallel with attention: GELU(h W_up^T + b) lands right of the attention columns
      PF_TRY(gemm(s, PF_KC_GEMM_UP, h, D, lw.w_up, D, lw.b_up, a + (size_t)D * e, D + F, RT, F, D, 0, 0, nullptr, nullptr, 0, nullptr, 0));
      PF_TRY(attention(s, PF_KC_ATTENTION, qkv, 3 * D, kb, vb, d.Lkv, d.Lp, a, D + F, R, q_pre));
      PF_TRY(gemm(s, PF_KC_GEMM_DOWN, a, D + F, lw.w_down, D + F, lw.b_down, xbuf, D, RT, D, D + F, 1, 0, m + 2 * D, xsrc, D, nullptr, 0, nullptr, R));
      xsrc = xbuf;
      continue;
    }

    // kinds 0, 1, 2: streams = [text (kind 2, if present), image]; r0 = first residual row, seg = rows per image
    struct Stream { const pf_layer_weights *lw; const float *m; size_t r0; int seg, brow0; };
    Stream streams[2];
    int ns = 0;
    if (c.kind == PF_BLOCK_MMDIT_JOINT && Tt) streams[ns++] = Stream{&s->txt[l], s->mod(0, l), t_row0, Tt, 0};
    streams[ns++] = Stream{&s->img[l], s->mod(d.n_streams - 1, l), Tt ? i_row0 : 0, n_img, row0_img};

    // final joint block: the text rows (first stream) are projected to keys and values and nothing else
    const bool txt_kv_only = c.txt_pre_only_last && l == c.n_layers - 1 && ns == 2;
    // q is handed over with the attention kernel's factor folded in only if every stream's projection rewrites q in fp32
    q_pre = pre_ok;
    for (int si = 0; si < ns && q_pre; ++si) {
      const Stream &sm = streams[si];
      const bool rot = d.rope && sm.lw == &s->img[l];
      q_pre = qkv_route(s, h + sm.r0 * D * e, *sm.lw, qkv + sm.r0 * 3 * D * e, rot) != ROUTE_SCATTER_PLAIN;
    }
    for (int si = 0; si < ns; ++si) {
      const Stream &sm = streams[si];
      const float *xs = xsrc + sm.r0 * D;
      char *hs = h + sm.r0 * D * e;
      char *qs = qkv + sm.r0 * 3 * D * e;
      PF_TRY(run(s, PF_KC_LN_MODULATE, [&] { return launch_ln_modulate(dt, xs, D, sm.m, sm.m + D, c.ln_eps, hs, D, B * sm.seg, D, 1, st, B > 1 ? sm.seg : 0, mstride); }));
      const bool rot = d.rope && sm.lw == &s->img[l];   // image stream of a rotating two-stream block
      pf_status qs_ = qkv_project(s, hs, *sm.lw, qs, sm.seg, kb, vb, 0, 0, sm.brow0, rot ? ws + w.rope : nullptr,
                                  rot ? img_off : -1, rot, q_pre ? q_fold : 0.f);
      if (qs_ != PF_OK) return qs_;
    }
    if (B == 1 && !txt_kv_only) {
      // one image: the text and image rows are adjacent, one launch covers both
      PF_TRY(attention(s, PF_KC_ATTENTION, qkv, 3 * D, kb, vb, d.Lkv, d.Lp, a, D, R, q_pre));
    } else {
      for (int si = txt_kv_only ? 1 : 0; si < ns; ++si)
        PF_TRY(attention(s, PF_KC_ATTENTION, qkv + streams[si].r0 * 3 * D * e, 3 * D, kb, vb, d.Lkv, d.Lp,
                         a + streams[si].r0 * D * e, D, streams[si].seg, q_pre));
    }
    for (int si = txt_kv_only ? 1 : 0; si < ns; ++si) {
      const Stream &sm = streams[si];
      const int nr = B * sm.seg;
      float *xs = xbuf + sm.r0 * D;
      const float *xs_in = xsrc + sm.r0 * D;   // differs from xs only before the first update
      char *hs = h + sm.r0 * D * e;
      char *as = a + sm.r0 * D * e;
      char *us = u + sm.r0 * F * e;
      const bool xattn = c.kind == PF_BLOCK_ADALN_SINGLE_XATTN;
      char *xb = xattn ? ws + w.xb : nullptr;
      PF_TRY(gemm(s, PF_KC_GEMM_OUT, as, D, sm.lw->w_o, D, sm.lw->b_o, xs, D, nr, D, D, 1, 0, sm.m + 2 * D, xs_in, D, xb, D, nullptr, sm.seg));
      if (xattn) {
        char *qc = ws + w.qc;
        PF_TRY(gemm(s, PF_KC_GEMM_XATTN, xb, D, sm.lw->xattn_wq, D, sm.lw->xattn_bq, qc, D, nr, D, D, 0, D, nullptr, nullptr, 0, nullptr, 0));
        PF_TRY(attention(s, PF_KC_XATTN, qc, D, s->kcptr(l), s->vcptr(l), d.T, d.Tp, as, D, sm.seg));
        PF_TRY(gemm(s, PF_KC_GEMM_XATTN, as, D, sm.lw->xattn_wo, D, sm.lw->xattn_bo, xs, D, nr, D, D, 1, 0, nullptr, xs, D, nullptr, 0));
      }
      PF_TRY(run(s, PF_KC_LN_MODULATE, [&] { return launch_ln_modulate(dt, xs, D, sm.m + 3 * D, sm.m + 4 * D, c.ln_eps, hs, D, nr, D, 1, st, B > 1 ? sm.seg : 0, mstride); }));
      PF_TRY(gemm(s, PF_KC_GEMM_UP, hs, D, sm.lw->w_up, D, sm.lw->b_up, us, F, nr, F, D, 0, 0, nullptr, nullptr, 0, nullptr, 0));
      PF_TRY(gemm(s, PF_KC_GEMM_DOWN, us, F, sm.lw->w_down, F, sm.lw->b_down, xs, D, nr, D, F, 1, 0, sm.m + 5 * D, xs, D, nullptr, 0, nullptr, sm.seg));
    }
    xsrc = xbuf;   // every stream of this layer has written its rows
  }

  if (y_img && xbuf != y_img)
    PF_TRY(run(s, PF_KC_COPY, [&] { return copy_blocks(y_img, (size_t)n_img * D, xres + i_row0 * D, i_pitch * D, (size_t)n_img * D, B, st); }));
  if (Tt && text_out)
    PF_TRY(run(s, PF_KC_COPY, [&] { return copy_blocks(text_out, (size_t)Tt * D, xres + t_row0 * D, t_pitch * D, (size_t)Tt * D, B, st); }));
  return PF_OK;
}

}  // namespace

extern "C" {

size_t pf_stage_kv_bytes(const pf_config *cfg) {
  pf_status st;
  if (!cfg || check_config(cfg, &st)) return 0;
  Derived d = derive(cfg);
  return kv_layer_bytes(cfg, d) * cfg->n_layers;
}

size_t pf_stage_workspace_bytes(const pf_config *cfg) {
  pf_status st;
  if (!cfg || check_config(cfg, &st)) return 0;
  Derived d = derive(cfg);
  return ws_layout(cfg, d).total;
}

pf_status pf_stage_create(const pf_config *cfg, const pf_layer_weights *layers, void *kv_buffer, size_t kv_bytes,
                          void *workspace, size_t ws_bytes, void *hip_stream, pf_stage **out) {
  if (out) *out = nullptr;
  if (!cfg || !layers || !kv_buffer || !workspace || !out) return fail(nullptr, PF_ERR_NULL, "null argument to pf_stage_create");
  pf_status st;
  if (const char *msg = check_config(cfg, &st)) return fail(nullptr, st, msg);
  Derived d = derive(cfg);
  WsLayout w = ws_layout(cfg, d);
  if (kv_bytes < kv_layer_bytes(cfg, d) * cfg->n_layers) return fail(nullptr, PF_ERR_WORKSPACE, "kv buffer too small");
  if (ws_bytes < w.total) return fail(nullptr, PF_ERR_WORKSPACE, "workspace too small");
  if (((uintptr_t)kv_buffer & 255) || ((uintptr_t)workspace & 255)) return fail(nullptr, PF_ERR_WORKSPACE, "kv buffer and workspace must be 256-byte aligned");
  const int kind = cfg->kind;
  for (int l = 0; l < cfg->n_layers; ++l) {
    const pf_layer_weights *streams[2] = {&layers[l], kind == PF_BLOCK_MMDIT_JOINT ? layers[l].txt : nullptr};
    if (kind == PF_BLOCK_MMDIT_JOINT && !layers[l].txt) return fail(nullptr, PF_ERR_NULL, "kind 2 needs text-stream weights (txt)");
    for (const pf_layer_weights *lw : streams) {
      if (!lw) continue;
      // the text stream of a final joint block only produces keys and values
      const bool kv_only = cfg->txt_pre_only_last && l == cfg->n_layers - 1 && lw == streams[1];
      bool ok = lw->w_mod && lw->w_qkv && lw->b_qkv && (kv_only || (lw->w_up && lw->b_up && lw->w_down && lw->b_down));
      if (kind != PF_BLOCK_ADALN_SINGLE_XATTN) ok = ok && lw->b_mod;
      if (kind != PF_BLOCK_SINGLE_STREAM) ok = ok && (kv_only || (lw->w_o && lw->b_o));
      if (kind == PF_BLOCK_ADALN_SINGLE_XATTN)
        ok = ok && lw->xattn_wq && lw->xattn_bq && lw->xattn_wkv && lw->xattn_bkv && lw->xattn_wo && lw->xattn_bo;
      if (cfg->qk_norm) ok = ok && lw->q_norm_w && lw->k_norm_w;
      if (!ok) return fail(nullptr, PF_ERR_NULL, "a required weight pointer of layer " + std::to_string(l) + " is null");
    }
  }
  pf_stage *s = new pf_stage();
  s->cfg = *cfg; s->d = d; s->w = w;
  s->img.assign(layers, layers + cfg->n_layers);
  if (kind == PF_BLOCK_MMDIT_JOINT)
    for (int l = 0; l < cfg->n_layers; ++l) s->txt.push_back(*layers[l].txt);
  s->kv = (char *)kv_buffer; s->ws = (char *)workspace; s->stream = (hipStream_t)hip_stream;
  *out = s;
  g_create_error.clear();
  return PF_OK;
}

pf_status pf_kv_init(pf_stage *s, const float *x_prev, const pf_cond *cp, float *y_prev) {
  if (!s) return PF_ERR_NULL;
  const pf_config &c = s->cfg;
  const Derived &d = s->d;
  if (c.kind == PF_BLOCK_ADALN_SINGLE_XATTN && (!cp || !cp->text)) return fail(s, PF_ERR_NULL, "kind 1: pf_kv_init needs cond_prev->text");
  if (x_prev) {
    if (!cp || !cp->cond) return fail(s, PF_ERR_NULL, "warm-up pass needs cond_prev->cond");
    if (d.Tj && !cp->text) return fail(s, PF_ERR_NULL, "joint kinds: warm-up pass needs cond_prev->text");
  }
  s->err.clear();
  s->chain_open = false;   // other work may have been enqueued on the stream since the last call
  s->mod_valid[0] = s->mod_valid[1] = false;
  PF_TRY(run(s, PF_KC_COPY, [&] { return launch_fill_zero(s->kv, kv_layer_bytes(&c, d) * c.n_layers, s->stream); }));
  if (c.kind == PF_BLOCK_ADALN_SINGLE_XATTN) {
    // text keys/values of every layer's cross-attention, computed once
    const int D = c.hidden;
    char *qkv = s->ws + s->w.qkv;
    for (int l = 0; l < c.n_layers; ++l) {
      const pf_layer_weights &lw = s->img[l];
      // text features of all images, [B][T][cross_dim], in one GEMM; then one scatter per image
      PF_TRY(gemm(s, PF_KC_GEMM_XATTN, cp->text, c.cross_dim, lw.xattn_wkv, c.cross_dim, lw.xattn_bkv, qkv + (size_t)D * d.esz,
                  3 * D, d.B * d.T, 2 * D, c.cross_dim, 0, 2 * D, nullptr, nullptr, 0, nullptr, 0));
      for (int b = 0; b < d.B; ++b) {
        ScatterArgs sa{c.dtype, qkv + (size_t)b * d.T * 3 * D * d.esz, 3 * D, s->kcptr(l) + b * s->ximg_elems() * d.esz,
                       s->vcptr(l) + b * s->ximg_elems() * d.esz, d.Tp, c.n_heads, c.head_dim, 0, d.T, 0, -1, c.grid_w, c.rope_theta};
        PF_TRY(run(s, PF_KC_KV_SCATTER, [&] { return launch_kv_scatter(sa, s->stream); }));
      }
    }
  }
  if (x_prev) {
    pf_status st = forward(s, x_prev, c.seq_img, 0, cp->cond, d.Tj ? (const float *)cp->text : nullptr, y_prev,
                           d.Tj ? cp->text_out : nullptr);
    if (st != PF_OK) return st;
  }
  s->ready = true;
  return PF_OK;
}

pf_status pf_stage_patch_forward(pf_stage *s, const float *x_patch, const pf_cond *cond, int patch_idx, float *y_patch) {
  if (!s) return PF_ERR_NULL;
  if (!x_patch || !y_patch || !cond || (!cond->cond && !cond->same_cond)) return fail(s, PF_ERR_NULL, "null argument to pf_stage_patch_forward");
  if (!s->ready) return fail(s, PF_ERR_STATE, "pf_kv_init must run before pf_stage_patch_forward");
  if (patch_idx < 0 || patch_idx >= s->cfg.n_patches) return fail(s, PF_ERR_RANGE, "patch index out of range");
  const bool joint_text = s->d.Tj && cond->text;
  if (joint_text && !cond->text_out) return fail(s, PF_ERR_NULL, "text rows given without text_out");
  s->err.clear();
  s->chain_open = false;   // other work may have been enqueued on the stream since the last call
  return forward(s, x_patch, s->d.n, patch_idx * s->d.n, cond->cond, joint_text ? (const float *)cond->text : nullptr,
                 y_patch, joint_text ? cond->text_out : nullptr, cond->same_cond != 0);
}

static pf_status fill_view(const pf_stage *s, int layer, int image, bool cross, pf_kv_view_t *out) {
  if (!s || !out) return PF_ERR_NULL;
  if (layer < 0 || layer >= s->cfg.n_layers || image < 0 || image >= s->d.B) return PF_ERR_RANGE;
  if (cross && s->cfg.kind != PF_BLOCK_ADALN_SINGLE_XATTN) return PF_ERR_CONFIG;
  const int dh = s->cfg.head_dim;
  const int rp = cross ? s->d.Tp : s->d.Lp;
  const size_t ioff = (size_t)image * (cross ? s->ximg_elems() : s->img_elems()) * s->d.esz;
  out->k = (cross ? s->kcptr(layer) : s->kptr(layer)) + ioff;
  out->v = (cross ? s->vcptr(layer) : s->vptr(layer)) + ioff;
  out->rows = cross ? s->d.T : s->d.Lkv;
  out->rows_padded = rp;
  out->text_rows = cross ? 0 : s->d.Tj;
  out->elem_bytes = (int32_t)s->d.esz;
  out->k_row_stride = dh; out->k_head_stride = (int64_t)rp * dh; out->k_col_stride = 1;
  out->v_row_stride = 1; out->v_head_stride = (int64_t)dh * rp; out->v_col_stride = rp;
  return PF_OK;
}

pf_status pf_kv_view(const pf_stage *s, int layer, pf_kv_view_t *out) { return fill_view(s, layer, 0, false, out); }
pf_status pf_xattn_kv_view(const pf_stage *s, int layer, pf_kv_view_t *out) { return fill_view(s, layer, 0, true, out); }
pf_status pf_kv_view_image(const pf_stage *s, int layer, int image, int cross, pf_kv_view_t *out) {
  return fill_view(s, layer, image, cross != 0, out);
}

pf_status pf_stage_attention_plan(const pf_stage *s, int nq, int cross, int *splits, size_t *ws_needed,
                                  size_t *ws_reserved) {
  if (!s || !splits || !ws_needed || !ws_reserved) return PF_ERR_NULL;
  if (nq < 1 || nq > s->d.Lkv) return PF_ERR_RANGE;
  if (cross && s->cfg.kind != PF_BLOCK_ADALN_SINGLE_XATTN) return PF_ERR_CONFIG;
  *splits = plan_splits(s, nq, cross ? s->d.T : s->d.Lkv);
  *ws_needed = attention_ws_bytes(nq, s->cfg.n_heads * s->d.B, s->cfg.head_dim, *splits);
  *ws_reserved = s->w.attn_bytes;
  return PF_OK;
}

pf_status pf_stage_set_stream(pf_stage *s, void *hip_stream) {
  if (!s) return PF_ERR_NULL;
  s->stream = (hipStream_t)hip_stream;
  return PF_OK;
}

pf_status pf_stage_profile(pf_stage *s, int enable) {
  if (!s) return PF_ERR_NULL;
  s->prof = enable != 0;
  s->chain_open = false;
  return PF_OK;
}

pf_status pf_stage_profile_read(pf_stage *s, double *ms, int64_t *launches) {
  if (!s || !ms || !launches) return PF_ERR_NULL;
  for (int i = 0; i < PF_KC_COUNT; ++i) { ms[i] = 0.0; launches[i] = 0; }
  if (s->events.empty()) return PF_OK;
  PF_TRY(hipStreamSynchronize(s->stream));
  for (size_t i = 0; i < s->events.size(); ++i) {
    const pf_stage::Mark &m = s->events[i];
    float t = 0.f;
    if (m.cls >= 0 && i > 0 && hipEventElapsedTime(&t, s->events[i - 1].ev, m.ev) == hipSuccess) {
      ms[m.cls] += t;
      launches[m.cls] += 1;
    }
  }
  for (auto &m : s->events) s->pool.push_back(m.ev);
  s->events.clear();
  s->chain_open = false;
  return PF_OK;
}

void pf_stage_destroy(pf_stage *s) {
  if (!s) return;
  for (auto &m : s->events) (void)hipEventDestroy(m.ev);
  for (auto e : s->pool) (void)hipEventDestroy(e);
  delete s;
}

const char *pf_status_str(pf_status st) {
  switch (st) {
    case PF_OK: return "PF_OK";
    case PF_ERR_NULL: return "PF_ERR_NULL";
    case PF_ERR_CONFIG: return "PF_ERR_CONFIG";
    case PF_ERR_SHAPE: return "PF_ERR_SHAPE";
    case PF_ERR_DTYPE: return "PF_ERR_DTYPE";
    case PF_ERR_STATE: return "PF_ERR_STATE";
    case PF_ERR_RANGE: return "PF_ERR_RANGE";
    case PF_ERR_WORKSPACE: return "PF_ERR_WORKSPACE";
    case PF_ERR_DEVICE: return "PF_ERR_DEVICE";
  }
  return "PF_ERR_UNKNOWN";
}

const char *pf_last_error(const pf_stage *s) { return s ? s->err.c_str() : g_create_error.c_str(); }

// ---- single-operator entry points ---------------------------------------------------------------------------
static bool dt_ok(int dt) { return dt == PF_F32 || dt == PF_BF16; }
static bool al16(const void *p) { return ((uintptr_t)p & 15) == 0; }

pf_status pf_op_modulation(int dtype, const void *w, const void *b, const float *c, float *mod, int out_dim, int in_dim,
                           int table_mode, void *stream) {
  if (!w || !c || !mod || (!table_mode && !b)) return PF_ERR_NULL;
  if (!dt_ok(dtype)) return PF_ERR_DTYPE;
  if (out_dim < 1 || in_dim < 8 || in_dim % 8 || in_dim > 12288 || !al16(w)) return PF_ERR_SHAPE;
  return launch_modulation(dtype, w, b, c, mod, out_dim, in_dim, table_mode, (hipStream_t)stream) == hipSuccess ? PF_OK : PF_ERR_DEVICE;
}

pf_status pf_op_ln_modulate(int dtype, const float *x, int64_t ldx, const float *shift, const float *scale, float eps,
                            void *out, int64_t ldo, int rows, int d, int normalize, void *stream) {
  if (!x || !out || (normalize && (!shift || !scale))) return PF_ERR_NULL;
  if (!dt_ok(dtype)) return PF_ERR_DTYPE;
  if (rows < 0 || d < 8 || d % 8 || d > 8192 || ldx < d || ldo < d || ldx % 4 || ldo % 4 || !al16(x) || !al16(out)) return PF_ERR_SHAPE;
  return launch_ln_modulate(dtype, x, ldx, shift, scale, eps, out, ldo, rows, d, normalize, (hipStream_t)stream) == hipSuccess ? PF_OK : PF_ERR_DEVICE;
}

int pf_gemm_tile_map(int M, int N, int tile_m, int tile_n, unsigned workgroup, unsigned *grid, int *tm, int *tn) {
  if (!grid || !tm || !tn) return PF_ERR_NULL;
  if (M < 1 || N < 1 || tile_m < 1 || tile_n < 1) return PF_ERR_RANGE;
  *tm = *tn = -1;
  return pf::gemm_tile_map(M, N, tile_m, tile_n, workgroup, grid, tm, tn) ? 1 : 0;
}

int pf_gemm_tile_count(void) { return gemm_mfma_dl_tile_count(); }

pf_status pf_op_gemm(int dtype, int path, const void *A, int64_t lda, const void *W, int64_t ldw, const void *bias, void *C,
                     int64_t ldc, int M, int N, int K, int epilogue, int gelu_from, int gelu_tanh, const float *gate,
                     const float *R, int64_t ldr, void *C2, int64_t ldc2, void *stream) {
  return pf_op_gemm_tile(0, dtype, path, A, lda, W, ldw, bias, C, ldc, M, N, K, epilogue, gelu_from, gelu_tanh, gate, R, ldr, C2,
                         ldc2, stream);
}

pf_status pf_op_gemm_tile(int tile, int dtype, int path, const void *A, int64_t lda, const void *W, int64_t ldw,
                          const void *bias, void *C, int64_t ldc, int M, int N, int K, int epilogue, int gelu_from,
                          int gelu_tanh, const float *gate, const float *R, int64_t ldr, void *C2, int64_t ldc2,
                          void *stream) {
  if (!A || !W || !C || (epilogue == 1 && !R)) return PF_ERR_NULL;
  if (tile < 0 || tile > gemm_mfma_dl_tile_count()) return PF_ERR_RANGE;
  if (tile > 0 && (dtype != PF_BF16 || path != PF_PATH_AUTO || K % 64)) return PF_ERR_SHAPE;   // tiles exist for the bf16 MFMA kernels
  if (!dt_ok(dtype)) return PF_ERR_DTYPE;
  if (M < 0 || N < 1 || K < 8 || K % 8 || lda < K || ldw < K || lda % 8 || ldw % 8 || ldc < N || !al16(A) || !al16(W)) return PF_ERR_SHAPE;
  if (epilogue != 0 && epilogue != 1) return PF_ERR_SHAPE;
  if (epilogue == 1 && ldr < N) return PF_ERR_SHAPE;
  if (C2 && ldc2 < N) return PF_ERR_SHAPE;
  GemmArgs g{};
  g.dt = dtype; g.path = (dtype == PF_BF16 && path == PF_PATH_AUTO) ? PATH_AUTO : PATH_SIMT;
  g.A = A; g.lda = lda; g.W = W; g.ldw = ldw; g.bias = bias; g.C = C; g.ldc = ldc; g.M = M; g.N = N; g.K = K;
  g.epilogue = epilogue; g.gelu_from = gelu_from; g.gelu_tanh = gelu_tanh; g.gate = gate; g.R = R; g.ldr = ldr; g.C2 = C2; g.ldc2 = ldc2;
  g.tile = tile;
  return launch_gemm(g, (hipStream_t)stream) == hipSuccess ? PF_OK : PF_ERR_DEVICE;
}

pf_status pf_op_kv_scatter(int dtype, void *qkv, int64_t ld, void *kbuf, void *vtbuf, int rows_padded, int n_heads,
                           int head_dim, int row0, int rows, int rope, int tok0, int grid_w, float rope_theta,
                           const void *q_norm_w, const void *k_norm_w, float norm_eps, void *stream) {
  if (!qkv || !kbuf || !vtbuf) return PF_ERR_NULL;
  if (!dt_ok(dtype)) return PF_ERR_DTYPE;
  const int64_t d = (int64_t)n_heads * head_dim;
  if (n_heads < 1 || head_dim < 8 || head_dim % 8 || ld < 3 * d || ld % 8 || rows < 0 || row0 < 0 ||
      (int64_t)row0 + rows > rows_padded || rows_padded % 8 || !al16(qkv) || !al16(kbuf) || !al16(vtbuf))
    return PF_ERR_SHAPE;
  if (rope && (head_dim % 4 || grid_w < 1 || !(rope_theta > 1.f))) return PF_ERR_SHAPE;
  if ((q_norm_w == nullptr) != (k_norm_w == nullptr)) return PF_ERR_NULL;
  if (q_norm_w && ((head_dim & (head_dim - 1)) || !(norm_eps >= 0.f) || !al16(q_norm_w) || !al16(k_norm_w))) return PF_ERR_SHAPE;
  ScatterArgs sa{dtype, qkv, ld, kbuf, vtbuf, rows_padded, n_heads, head_dim, row0, rows, rope, tok0, grid_w, rope_theta};
  sa.q_norm_w = q_norm_w; sa.k_norm_w = k_norm_w; sa.norm_eps = norm_eps;
  return launch_kv_scatter(sa, (hipStream_t)stream) == hipSuccess ? PF_OK : PF_ERR_DEVICE;
}

pf_status pf_op_axpy(const float *x, const float *y, float alpha, float *out, int64_t n, void *stream) {
  if (n < 0) return PF_ERR_SHAPE;
  if (n == 0) return PF_OK;
  if (!x || !y || !out) return PF_ERR_NULL;
  return launch_axpby(x, y, 1.0f, alpha, out, n, (hipStream_t)stream) == hipSuccess ? PF_OK : PF_ERR_DEVICE;
}

pf_status pf_op_axpby(const float *x, const float *y, float a, float b, float *out, int64_t n, void *stream) {
  if (n < 0) return PF_ERR_SHAPE;
  if (n == 0) return PF_OK;
  if (!x || !y || !out) return PF_ERR_NULL;
  return launch_axpby(x, y, a, b, out, n, (hipStream_t)stream) == hipSuccess ? PF_OK : PF_ERR_DEVICE;
}

const char *pf_gemm_kernel_name(int dtype, int path, int M, int N, int K) {
  GemmArgs g{};
  g.dt = dtype; g.path = (dtype == PF_BF16 && path == PF_PATH_AUTO) ? PATH_AUTO : PATH_SIMT; g.M = M; g.N = N; g.K = K;
  if (g.path == PATH_SIMT || dtype != PF_BF16) return "gemm_simt_kernel";
  return gemm_mfma_dl_supported(g) ? gemm_mfma_dl_variant_name(g) : "gemm_mfma_kernel";
}

const char *pf_attention_kernel_name(int dtype, int path, int head_dim, int nq, int q_prescaled) {
  if (dtype != PF_BF16 || path != PF_PATH_AUTO) return "attn_simt_kernel";
  if (pf::g_attn_variant != 0 || !(head_dim == 64 || head_dim == 72 || head_dim == 128)) return "attn_mfma_kernel";
  static thread_local char name[64];
  const bool wide = attn_mfma2_qtile(nq) == 256;
  const int ns = wide ? 4 : (pf::g_attn_stages ? pf::g_attn_stages : 2);
  snprintf(name, sizeof(name), "attn_mfma2_kernel<%d,%d,%s,%d>", head_dim, ns, q_prescaled ? "true" : "false", wide ? 8 : 4);
  return name;
}

pf_status pf_probe_mfma_loop(float *out, int workgroups, int iters, double *flops, void *stream) {
  if (!out || !flops) return PF_ERR_NULL;
  if (workgroups < 1 || workgroups > 65536 || iters < 1) return PF_ERR_SHAPE;
  *flops = (double)workgroups * 4.0 * (double)iters * 32.0 * 32768.0;
  return launch_mfma_loop(out, workgroups, iters, (hipStream_t)stream) == hipSuccess ? PF_OK : PF_ERR_DEVICE;
}

size_t pf_op_attention_ws_bytes(int nq, int n_heads, int head_dim, int splits) {
  return attention_ws_bytes(nq, n_heads, head_dim, splits);
}

static pf_status attention_args_check(int dtype, const void *q, int64_t ldq, const void *kbuf, const void *vtbuf, int kv_rows,
                                      int rows_padded, int n_heads, int head_dim, const void *out, int64_t ldo, int nq,
                                      int splits) {
  if (!q || !kbuf || !vtbuf || !out) return PF_ERR_NULL;
  if (!dt_ok(dtype)) return PF_ERR_DTYPE;
  const int64_t d = (int64_t)n_heads * head_dim;
  if (n_heads < 1 || head_dim < 8 || head_dim % 8 || head_dim > 128 || kv_rows < 1 || rows_padded % 128 || kv_rows > rows_padded ||
      ldq < d || ldo < d || ldq % 8 || ldo % 4 || nq < 0 || splits < 1 || splits > 64 || !al16(q) || !al16(kbuf) || !al16(vtbuf) || ((uintptr_t)out & 7))
    return PF_ERR_SHAPE;
  return PF_OK;
}

static pf_status attention_launch(int dtype, int path, const void *q, int64_t ldq, const void *kbuf, const void *vtbuf,
                                  int kv_rows, int rows_padded, int n_heads, int head_dim, void *out, int64_t ldo, int nq,
                                  int splits, float *ws, hipStream_t st) {
  AttnArgs a{};
  const bool prescaled = path == PF_PATH_AUTO_PRESCALED_Q;
  a.dt = dtype; a.path = (dtype == PF_BF16 && (path == PF_PATH_AUTO || prescaled)) ? PATH_AUTO : PATH_SIMT;
  a.q_prescaled = prescaled ? 1 : 0;
  a.q = q; a.ldq = ldq; a.kbuf = kbuf; a.vtbuf = vtbuf; a.kv_rows = kv_rows; a.rows_padded = rows_padded; a.n_heads = n_heads;
  a.head_dim = head_dim; a.out = out; a.ldo = ldo; a.nq = nq; a.splits = splits; a.ws = ws;
  if (prescaled && (dtype != PF_BF16 || !pf::attn_mfma2_takes_prescaled_q(head_dim) || !pf::attn_mfma2_supported(a) || pf::g_attn_variant != 0))
    return fail(nullptr, PF_ERR_SHAPE, "PF_PATH_AUTO_PRESCALED_Q needs bf16 and head_dim 64, 72 or 128");
  hipError_t e = a.path == PATH_SIMT ? launch_attn_simt(a, st) : launch_attn_bf16(a, st);
  if (e == hipSuccess && splits > 1) e = launch_attn_combine(a, st);
  return e == hipSuccess ? PF_OK : PF_ERR_DEVICE;
}

pf_status pf_op_attention(int dtype, int path, const void *q, int64_t ldq, const void *kbuf, const void *vtbuf, int kv_rows,
                          int rows_padded, int n_heads, int head_dim, void *out, int64_t ldo, int nq, int splits, void *ws,
                          size_t ws_bytes, void *stream) {
  pf_status st = attention_args_check(dtype, q, ldq, kbuf, vtbuf, kv_rows, rows_padded, n_heads, head_dim, out, ldo, nq, splits);
  if (st != PF_OK) return st;
  if (splits > 1 && (!ws || ws_bytes < attention_ws_bytes(nq, n_heads, head_dim, splits) || !al16(ws))) return PF_ERR_WORKSPACE;
  return attention_launch(dtype, path, q, ldq, kbuf, vtbuf, kv_rows, rows_padded, n_heads, head_dim, out, ldo, nq, splits,
                          (float *)ws, (hipStream_t)stream);
}

// ---- the entry point that allocates nothing ------------------------------------------------------------------
// Split-KV partial results of pf_op_attention_static live in this array instead of a caller-provided workspace.  Every
// GPU the library runs on holds its own copy at its own address for the life of the process; host code never uses the
// array's name as an address, only the per-device pointer that hipGetSymbolAddress returned.
static __device__ __align__(256) unsigned char scratch[PF_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` per device ordinal, filled on first use

// Device address of this device's copy of `scratch` (the current device's; looked up once per device).
pf_status static_scratch(void **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return PF_ERR_DEVICE;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return PF_ERR_DEVICE;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return PF_OK;
}
}  // namespace

size_t pf_static_scratch_bytes(void) { return PF_STATIC_SCRATCH_BYTES; }

pf_status pf_op_attention_static(int dtype, int path, const void *q, int64_t ldq, const void *kbuf, const void *vtbuf,
                                 int kv_rows, int rows_padded, int n_heads, int head_dim, void *out, int64_t ldo, int nq,
                                 int splits, void *stream) {
  pf_status st = attention_args_check(dtype, q, ldq, kbuf, vtbuf, kv_rows, rows_padded, n_heads, head_dim, out, ldo, nq, splits);
  if (st != PF_OK) return st;
  const size_t need = attention_ws_bytes(nq, n_heads, head_dim, splits);
  if (need > PF_STATIC_SCRATCH_BYTES)
    return fail(nullptr, PF_ERR_WORKSPACE,
                "pf_op_attention_static: the split partial results need " + std::to_string(need) + " bytes, the static scratch array holds " +
                    std::to_string((size_t)PF_STATIC_SCRATCH_BYTES) + "; use fewer splits or query rows, or pf_op_attention with a workspace");
  void *ws = nullptr;
  if (splits > 1) {
    st = static_scratch(&ws);
    if (st != PF_OK) return fail(nullptr, st, "pf_op_attention_static: no device address for the static scratch array");
  }
  // Nothing in the array has to start at zero: the attention launch writes every (split, query, head) slot that the
  // combine launch of the same call reads, so an earlier call's leftovers are never read.
  return attention_launch(dtype, path, q, ldq, kbuf, vtbuf, kv_rows, rows_padded, n_heads, head_dim, out, ldo, nq, splits,
                          (float *)ws, (hipStream_t)stream);
}

}  // extern "C"

namespace pf {
hipError_t launch_attn_bf16(const AttnArgs &a, hipStream_t s) {
  return (g_attn_variant == 0 && attn_mfma2_supported(a)) ? launch_attn_mfma2(a, s) : launch_attn_mfma(a, s);
}
hipError_t launch_gemm(const GemmArgs &a, hipStream_t s) {
  if (a.path == PATH_SIMT || a.dt != DT_BF16) return launch_gemm_simt(a, s);
  return gemm_mfma_dl_supported(a) ? launch_gemm_mfma_dl(a, s) : launch_gemm_mfma(a, s);
}
}  // namespace pf
