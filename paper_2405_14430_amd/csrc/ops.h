// Internal launch interface between the stage runtime (stage.cpp) and the kernel files.
// Every function only enqueues work on `s` and returns the launch status; shapes are validated
// by the callers (the C-ABI layer) before these are reached.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace pf {

enum { DT_F32 = 0, DT_BF16 = 1 };
enum { PATH_AUTO = 0, PATH_SIMT = 1 };

inline size_t dt_size(int dt) { return dt == DT_BF16 ? 2 : 4; }

// Launch-plan constants.  In the library as shipped they are compile-time constants: no process-wide state can change
// the plan of a live stage.  A build with -DPF_TUNING (tile and split sweeps on the GPU, never the shipped library)
// turns them into variables behind pf_tune(), declared in tuning.h.
#ifdef PF_TUNING
#define PF_PLAN_CONST(name, value) extern int name
#else
#define PF_PLAN_CONST(name, value) constexpr int name = value
#endif
PF_PLAN_CONST(g_attn_variant, 0);       // 0 = newest attention kernel that supports the shape, 1 = first-generation kernel
PF_PLAN_CONST(g_attn_stages, 0);        // attention ring depth: 0 = default, 2 / 3 = forced (4-wave kernel)
PF_PLAN_CONST(g_attn_wide, 0);          // 0 = 256-query workgroups when the launch has enough queries, 1 = never, 2 = always
PF_PLAN_CONST(g_force_splits, 0);       // > 0 replaces the split heuristic's count (still capped by the key tiles)
PF_PLAN_CONST(g_fuse_kv_route, 1);      // K/V written by the QKV GEMM epilogue (1) or by the scatter kernel (0)
PF_PLAN_CONST(g_fold_q_scale, 1);       // q reaches the attention kernel with its exponent factor folded in
PF_PLAN_CONST(g_gemm_tile_override, 0); // 0 = tile heuristic, else a fixed tile configuration for every launch
PF_PLAN_CONST(g_wavek_min_k, 2048);     // smallest K the wave-split-K GEMM kernel takes
PF_PLAN_CONST(g_wavek_max_tiles, 512);  // it takes GEMMs with fewer 64 x 64 tiles than this

hipError_t launch_modulation(int dt, const void *w, const void *b, const float *c, float *mod, int out_dim,
                             int in_dim, int table_mode, hipStream_t s);

// Up to kMax modulation vectors (layers x streams x images) in one launch; all share the shapes.
struct ModBatch {
  static constexpr int kMax = 16;
  const void *w[kMax];
  const void *b[kMax];
  const float *c[kMax];   // conditioning vector of the entry (differs per image of a batch)
  float *out[kMax];
  int count;
};
hipError_t launch_modulation_batch(int dt, const ModBatch &mb, int out_dim, int in_dim, int table_mode, hipStream_t s);

// seg_rows > 0: rows are image-major with seg_rows rows per image and image b reads its shift / scale vectors
// seg_stride floats after image 0's.
hipError_t launch_ln_modulate(int dt, const float *x, int64_t ldx, const float *shift, const float *scale,
                              float eps, void *out, int64_t ldo, int rows, int d, int normalize,
                              hipStream_t s, int seg_rows = 0, int64_t seg_stride = 0);

struct KvRoute;   // epilogue.h
// seg > 0: GEMM rows are image-major, seg per image; image b writes into kbuf / vtbuf + b * img_stride elements and
// the row mapping (split, row0a, row0b, rope row) applies to the row index inside the image.
struct GemmArgsKv { void *kbuf, *vtbuf; int Lp, dh, d, split, row0a, row0b; const void *rope; int seg; int64_t img_stride;
                    float q_scale; };   // q_scale != 0: the q columns are multiplied by it before they are rounded

struct GemmArgs {
  int dt, path;
  const void *A; int64_t lda;
  const void *W; int64_t ldw;
  const void *bias;
  void *C; int64_t ldc;
  int M, N, K;
  int epilogue;        // 0: store dtype (+GELU from column gelu_from); 1: fp32 residual update
  int gelu_from, gelu_tanh;
  const float *gate;   // [N] or nullptr
  int gate_seg; int64_t gate_stride;   // gate_seg > 0: row r uses gate + (r / gate_seg) * gate_stride (image-major rows)
  const float *R; int64_t ldr;
  void *C2; int64_t ldc2;
  GemmArgsKv kvr;      // kbuf == nullptr: plain GEMM
  int tile;            // 0: the tile heuristic picks; 1 .. gemm_mfma_dl_tile_count(): that tile configuration, this launch only
};
hipError_t launch_gemm(const GemmArgs &a, hipStream_t s);
bool gemm_kv_route_supported(const GemmArgs &a);   // the fused QKV -> K/V^T write needs the vectorised bf16 epilogue

// (cos, sin) of the RoPE angles for the rows of a call: rows [0, n_text) are text (no rotation), row n_text + i is image
// token tok0 + i on a grid of width grid_w.  tab is float2 [rows][dh/2].
hipError_t launch_rope_table(void *tab, int rows, int n_text, int tok0, int grid_w, int dh, float theta, hipStream_t s);

struct ScatterArgs {
  int dt;
  void *qkv; int64_t ld;
  void *kbuf, *vtbuf;
  int rows_padded, n_heads, head_dim, row0, rows;
  int rope, tok0, grid_w; float theta;
  const void *q_norm_w, *k_norm_w;   // [head_dim] scales of the per-head RMSNorm of q and k (before RoPE), or nullptr
  float norm_eps;
  float q_scale;                     // != 0 (needs rope or norm: q is rewritten anyway): q is multiplied by it
};
hipError_t launch_kv_scatter(const ScatterArgs &a, hipStream_t s);

struct AttnArgs {
  int dt, path;
  const void *q; int64_t ldq;
  const void *kbuf, *vtbuf;
  int kv_rows, rows_padded, n_heads, head_dim;
  void *out; int64_t ldo;
  int nq, splits;
  float *ws;           // partial results when splits > 1
  int q_prescaled;     // q already carries the factor log2(e) / sqrt(head_dim) (bf16 direct-to-LDS kernel only)
  int batch;           // images per call (0 or 1: one).  q / out hold batch x nq rows, image-major; kbuf / vtbuf hold
                       // batch x n_heads heads, image-major; the workspace is sized for n_heads * batch heads
};
size_t attention_ws_bytes(int nq, int n_heads, int head_dim, int splits);
hipError_t launch_attention(const AttnArgs &a, hipStream_t s, bool *used_combine);

hipError_t launch_axpby(const float *x, const float *y, float a, float b, float *out, int64_t n, hipStream_t s);
hipError_t launch_mfma_loop(float *out, int workgroups, int iters, hipStream_t s);   // measurement aid (probe.hip)
hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t s);   // bytes multiple of 16, p 16-byte aligned

// kernel-path specific pieces (defined in gemm_*.hip / attn_*.hip)
hipError_t launch_gemm_simt(const GemmArgs &a, hipStream_t s);
hipError_t launch_gemm_mfma(const GemmArgs &a, hipStream_t s);
bool gemm_tile_map(int M, int N, int BM, int BN, unsigned id, unsigned *grid, int *tm, int *tn);   // host view of the tile map
bool gemm_mfma_dl_supported(const GemmArgs &a);            // direct-to-LDS multi-stage variant (K % 64 == 0)
hipError_t launch_gemm_mfma_dl(const GemmArgs &a, hipStream_t s);
const char *gemm_mfma_dl_variant_name(const GemmArgs &a);   // kernel instance the tile heuristic picks for this shape
int gemm_mfma_dl_tile_count();                              // tile configurations the heuristic chooses from
hipError_t launch_attn_simt(const AttnArgs &a, hipStream_t s);
hipError_t launch_attn_mfma(const AttnArgs &a, hipStream_t s);
bool attn_partials_half(const AttnArgs &a);               // the launch for `a` leaves normalised fp16 partial outputs
bool attn_mfma2_supported(const AttnArgs &a);              // direct-to-LDS variant for head sizes 64 / 72 / 128
hipError_t launch_attn_mfma2(const AttnArgs &a, hipStream_t s);
int attn_mfma2_qtile(int nq);                              // queries per workgroup it will use for nq query rows per image
bool attn_mfma2_takes_prescaled_q(int head_dim);           // its kernel for this head size has a prescaled-q variant
hipError_t launch_attn_bf16(const AttnArgs &a, hipStream_t s);   // picks between the two
hipError_t launch_attn_combine(const AttnArgs &a, hipStream_t s);

}  // namespace pf
