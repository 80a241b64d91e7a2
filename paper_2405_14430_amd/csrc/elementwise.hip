// Streaming (HBM-bound) kernels of the patch stage: modulation vectors, LayerNorm + adaLN modulate,
// the K/V scatter into the full-sequence buffers (PipeFusion Sec. 3.3: fresh rows of the current patch
// replace the stale ones before attention), the split-KV combine, and a zero fill.
#include "common.h"
#include "ops.h"

namespace pf {

// ------------------------------------------------------------------------------------------------
// modulation: mod = W * SiLU(c) + b   (one wave per output), or mod = table + c
// ------------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void modulation_body(const T *__restrict__ w, const T *__restrict__ b,
                                                const float *__restrict__ c, float *__restrict__ mod, int out_dim,
                                                int in_dim, int table_mode);

template <typename T>
__global__ __launch_bounds__(256) void modulation_kernel(const T *__restrict__ w, const T *__restrict__ b,
                                                         const float *__restrict__ c, float *__restrict__ mod,
                                                         int out_dim, int in_dim, int table_mode) {
  modulation_body<T>(w, b, c, mod, out_dim, in_dim, table_mode);
}

// blockIdx.y selects the (layer, stream) entry
template <typename T>
__global__ __launch_bounds__(256) void modulation_batch_kernel(ModBatch mb, int out_dim, int in_dim, int table_mode) {
  const int e = blockIdx.y;
  modulation_body<T>((const T *)mb.w[e], (const T *)mb.b[e], mb.c[e], mb.out[e], out_dim, in_dim, table_mode);
}

template <typename T>
__device__ __forceinline__ void modulation_body(const T *__restrict__ w, const T *__restrict__ b,
                                                const float *__restrict__ c, float *__restrict__ mod, int out_dim,
                                                int in_dim, int table_mode) {
  if (table_mode) {
    int j = blockIdx.x * 256 + threadIdx.x;
    if (j < out_dim) mod[j] = to_f32(w[j]) + c[j];
    return;
  }
  extern __shared__ float sc[];  // SiLU(c), in_dim floats
  for (int i = threadIdx.x; i < in_dim; i += 256) sc[i] = silu_f(c[i]);
  __syncthreads();
  constexpr int V = Vec16<T>::N;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // 8 outputs per wave, 32 per block.  The eight weight rows are read side by side (eight 16-byte loads per lane in
  // flight per step instead of one row after the other): the kernel is a stream over the [out_dim, in_dim] weights.
  const int j0 = blockIdx.x * 32 + wave * 8;
  if (j0 >= out_dim) return;
  const T *rows[8];
#pragma unroll
  for (int o = 0; o < 8; ++o) rows[o] = w + (size_t)min(j0 + o, out_dim - 1) * in_dim;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int i = lane * V; i < in_dim; i += 64 * V) {
    float v[8][V];
#pragma unroll
    for (int o = 0; o < 8; ++o) Vec16<T>::load(rows[o] + i, v[o]);
#pragma unroll
    for (int o = 0; o < 8; ++o)
#pragma unroll
      for (int t = 0; t < V; ++t) acc[o] = fmaf(v[o][t], sc[i + t], acc[o]);
  }
#pragma unroll
  for (int o = 0; o < 8; ++o) acc[o] = wave_sum(acc[o]);
  if (lane == 0) {
#pragma unroll
    for (int o = 0; o < 8; ++o)
      if (j0 + o < out_dim) mod[j0 + o] = acc[o] + to_f32(b[j0 + o]);
  }
}

hipError_t launch_modulation_batch(int dt, const ModBatch &mb, int out_dim, int in_dim, int table_mode, hipStream_t s) {
  if (mb.count <= 0) return hipSuccess;
  dim3 g(table_mode ? (out_dim + 255) / 256 : (out_dim + 31) / 32, mb.count);
  size_t sh = table_mode ? 0 : (size_t)in_dim * sizeof(float);
  if (dt == DT_BF16) modulation_batch_kernel<bf16_t><<<g, 256, sh, s>>>(mb, out_dim, in_dim, table_mode);
  else modulation_batch_kernel<float><<<g, 256, sh, s>>>(mb, out_dim, in_dim, table_mode);
  return hipGetLastError();
}

hipError_t launch_modulation(int dt, const void *w, const void *b, const float *c, float *mod, int out_dim,
                             int in_dim, int table_mode, hipStream_t s) {
  if (table_mode) {
    dim3 g((out_dim + 255) / 256);
    if (dt == DT_BF16)
      modulation_kernel<bf16_t><<<g, 256, 0, s>>>((const bf16_t *)w, nullptr, c, mod, out_dim, in_dim, 1);
    else
      modulation_kernel<float><<<g, 256, 0, s>>>((const float *)w, nullptr, c, mod, out_dim, in_dim, 1);
  } else {
    dim3 g((out_dim + 31) / 32);
    size_t sh = (size_t)in_dim * sizeof(float);
    if (dt == DT_BF16)
      modulation_kernel<bf16_t><<<g, 256, sh, s>>>((const bf16_t *)w, (const bf16_t *)b, c, mod, out_dim, in_dim, 0);
    else
      modulation_kernel<float><<<g, 256, sh, s>>>((const float *)w, (const float *)b, c, mod, out_dim, in_dim, 0);
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// LayerNorm + modulate: WPR waves per row (1, 2 or 4), the row lives in registers (single pass over HBM).  One wave
// per row when there are rows enough to fill the chip with memory requests; fewer rows (a patch of 512 or 2048 tokens
// is only that many waves) are split over two or four waves each, which exchange their partial sums through LDS.
// NC = float4 chunks per lane; d <= NC * 256 * WPR.
// ------------------------------------------------------------------------------------------------
template <typename T, int NC, int WPR>
__global__ __launch_bounds__(256) void ln_modulate_kernel(const float *__restrict__ x, int64_t ldx,
                                                          const float *__restrict__ shift,
                                                          const float *__restrict__ scale, float eps,
                                                          T *__restrict__ out, int64_t ldo, int rows, int d,
                                                          int normalize, int seg_rows, int64_t seg_stride) {
  // rows are image-major, seg_rows per image; image b uses shift + b * seg_stride, scale + b * seg_stride
  constexpr int RPB = 4 / WPR;                       // rows per block
  __shared__ float part[2][4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wir = wave % WPR;                        // this wave's index inside its row
  const int row = blockIdx.x * RPB + wave / WPR;
  const bool live = row < rows;                      // (waves of a dead row still meet the barriers)
  if (live && seg_rows > 0) {
    const int64_t o = (int64_t)(row / seg_rows) * seg_stride;
    shift += o;
    scale += o;
  }
  const float *xr = x + (size_t)(live ? row : 0) * ldx;
  float4 v[NC];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NC; ++i) {
    int c = ((i * WPR + wir) * 64 + lane) * 4;
    if (live && c < d) {
      v[i] = *reinterpret_cast<const float4 *>(xr + c);
      sum += (v[i].x + v[i].y) + (v[i].z + v[i].w);
    } else {
      v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
  // sum over the row: within the wave, then over the row's WPR waves (fixed order: the result does not depend on timing)
  auto row_sum = [&](float s, int slot) -> float {
    s = wave_sum(s);
    if constexpr (WPR == 1) return s;
    if (lane == 0) part[slot][wave] = s;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < WPR; ++w) t += part[slot][(wave / WPR) * WPR + w];
    return t;
  };
  float mean = 0.f, rstd = 1.f;
  if (normalize) {
    mean = row_sum(sum, 0) / (float)d;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      int c = ((i * WPR + wir) * 64 + lane) * 4;
      if (c < d) {
        float a = v[i].x - mean, b = v[i].y - mean, e = v[i].z - mean, f = v[i].w - mean;
        sq += (a * a + b * b) + (e * e + f * f);
      }
    }
    rstd = rsqrtf(row_sum(sq, 1) / (float)d + eps);
  }
  if (!live) return;
  T *orow = out + (size_t)row * ldo;
#pragma unroll
  for (int i = 0; i < NC; ++i) {
    int c = ((i * WPR + wir) * 64 + lane) * 4;
    if (c < d) {
      float y[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
      if (normalize) {
        float4 sh = *reinterpret_cast<const float4 *>(shift + c);
        float4 sc = *reinterpret_cast<const float4 *>(scale + c);
        y[0] = (y[0] - mean) * rstd * (1.f + sc.x) + sh.x;
        y[1] = (y[1] - mean) * rstd * (1.f + sc.y) + sh.y;
        y[2] = (y[2] - mean) * rstd * (1.f + sc.z) + sh.z;
        y[3] = (y[3] - mean) * rstd * (1.f + sc.w) + sh.w;
      }
      if constexpr (sizeof(T) == 4) {
        *reinterpret_cast<float4 *>(orow + c) = make_float4(y[0], y[1], y[2], y[3]);
      } else {
        bf16x4 o;
        o[0] = (bf16_t)y[0]; o[1] = (bf16_t)y[1]; o[2] = (bf16_t)y[2]; o[3] = (bf16_t)y[3];
        *reinterpret_cast<bf16x4 *>(orow + c) = o;
      }
    }
  }
}

template <typename T, int NC, int WPR>
static void ln_launch(const float *x, int64_t ldx, const float *shift, const float *scale, float eps, void *out,
                      int64_t ldo, int rows, int d, int normalize, int seg_rows, int64_t seg_stride, hipStream_t s) {
  constexpr int RPB = 4 / WPR;
  ln_modulate_kernel<T, NC, WPR><<<dim3((rows + RPB - 1) / RPB), 256, 0, s>>>(x, ldx, shift, scale, eps, (T *)out, ldo, rows, d,
                                                                          normalize, seg_rows, seg_stride);
}

template <typename T, int WPR>
static hipError_t ln_dispatch_wpr(const float *x, int64_t ldx, const float *shift, const float *scale, float eps,
                                  void *out, int64_t ldo, int rows, int d, int normalize, int seg_rows, int64_t seg_stride,
                                  hipStream_t s) {
  int need = (d + 256 * WPR - 1) / (256 * WPR);
#define PF_LN_CASE(NC) \
  if (need <= NC) { ln_launch<T, NC, WPR>(x, ldx, shift, scale, eps, out, ldo, rows, d, normalize, seg_rows, seg_stride, s); return hipGetLastError(); }
  PF_LN_CASE(1) PF_LN_CASE(2) PF_LN_CASE(3) PF_LN_CASE(4) PF_LN_CASE(5) PF_LN_CASE(6) PF_LN_CASE(8) PF_LN_CASE(12) PF_LN_CASE(16) PF_LN_CASE(32)
#undef PF_LN_CASE
  return hipErrorInvalidValue;  // d > 8192 is rejected by the caller
}

template <typename T>
static hipError_t ln_dispatch(const float *x, int64_t ldx, const float *shift, const float *scale, float eps,
                              void *out, int64_t ldo, int rows, int d, int normalize, int seg_rows, int64_t seg_stride,
                              hipStream_t s) {
  // one wave per row needs about 8192 rows to keep every CU busy with memory requests (32 waves per CU); below that
  // the rows are split (a row of fewer than 512 floats is not worth splitting)
  const int wpr = (rows >= 8192 || d < 512) ? 1 : ((rows >= 4096 || d < 1024) ? 2 : 4);
  if (wpr == 4) return ln_dispatch_wpr<T, 4>(x, ldx, shift, scale, eps, out, ldo, rows, d, normalize, seg_rows, seg_stride, s);
  if (wpr == 2) return ln_dispatch_wpr<T, 2>(x, ldx, shift, scale, eps, out, ldo, rows, d, normalize, seg_rows, seg_stride, s);
  return ln_dispatch_wpr<T, 1>(x, ldx, shift, scale, eps, out, ldo, rows, d, normalize, seg_rows, seg_stride, s);
}

hipError_t launch_ln_modulate(int dt, const float *x, int64_t ldx, const float *shift, const float *scale,
                              float eps, void *out, int64_t ldo, int rows, int d, int normalize, hipStream_t s,
                              int seg_rows, int64_t seg_stride) {
  if (rows <= 0) return hipSuccess;
  return dt == DT_BF16 ? ln_dispatch<bf16_t>(x, ldx, shift, scale, eps, out, ldo, rows, d, normalize, seg_rows, seg_stride, s)
                       : ln_dispatch<float>(x, ldx, shift, scale, eps, out, ldo, rows, d, normalize, seg_rows, seg_stride, s);
}

// ------------------------------------------------------------------------------------------------
// K/V scatter (+ optional RoPE on q and k).
//   blocks [0, nbk): one thread per 16-byte chunk of the q and k parts of a row.  k chunks are copied to
//     K[h][row0+i][c..]; with rope both q and k chunks are rotated, written back in place, and the rotated
//     k goes to the buffer.
//   blocks [nbk, nbk+nbv): 64x64 (rows x channels) tiles of v transposed through LDS into V^T[h][c][row0+i].
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void kv_scatter_kernel(T *__restrict__ qkv, int64_t ld, T *__restrict__ kbuf,
                                                         T *__restrict__ vtbuf, int Lp, int H, int dh, int row0,
                                                         int rows, int rope, int tok0, int grid_w, float theta,
                                                         int nbk, const T *__restrict__ q_norm_w,
                                                         const T *__restrict__ k_norm_w, float norm_eps, float q_scale) {
  constexpr int V = Vec16<T>::N;
  const int d = H * dh;
  const bool norm = q_norm_w != nullptr;
  const bool inplace = rope || norm;   // q and k are rewritten in qkv (normalised and / or rotated)
  if ((int)blockIdx.x < nbk) {
    const int cpr = d / V;  // chunks per row per part
    const int parts = inplace ? 2 : 1;
    int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= (int64_t)rows * parts * cpr) return;
    int i = (int)(id / (parts * cpr));
    int rem = (int)(id % (parts * cpr));
    int part = inplace ? rem / cpr : 1;  // 0 = q, 1 = k
    int ch = (rem % cpr) * V;         // channel within the part
    T *src = qkv + (size_t)i * ld + (size_t)part * d + ch;
    float v[V];
    Vec16<T>::load(src, v);
    int h = ch / dh, c = ch % dh;
    if (norm) {
      // RMSNorm over the head's dh channels: they sit in dh / V consecutive lanes (a power of two, aligned)
      float ss = 0.f;
#pragma unroll
      for (int t = 0; t < V; ++t) ss = fmaf(v[t], v[t], ss);
      for (int m = 1; m < dh / V; m <<= 1) ss += __shfl_xor(ss, m, 64);
      const float rinv = rsqrtf(ss / (float)dh + norm_eps);
      const T *wn = (part == 0 ? q_norm_w : k_norm_w) + c;
#pragma unroll
      for (int t = 0; t < V; ++t) v[t] = v[t] * rinv * to_f32(wn[t]);
    }
    if (rope && tok0 >= 0) {
      int tok = tok0 + i;
      float pr = (float)(tok / grid_w), pc = (float)(tok % grid_w);
      int quarter = dh / 4;  // pairs per axis
#pragma unroll
      for (int t = 0; t < V; t += 2) {
        int j = (c + t) >> 1;  // pair index within the head
        int ia = j < quarter ? j : j - quarter;
        float pos = j < quarter ? pr : pc;
        // frequency theta^(-2*ia / (dh/2))
        float freq = exp2f(-log2f(theta) * (4.0f * (float)ia / (float)dh));
        float sn, cs;
        sincosf(pos * freq, &sn, &cs);
        float a = v[t], b = v[t + 1];
        v[t] = a * cs - b * sn;
        v[t + 1] = a * sn + b * cs;
      }
    }
    if (inplace) {
      if (part == 0 && q_scale != 0.f) {
#pragma unroll
        for (int t = 0; t < V; ++t) v[t] *= q_scale;
      }
      Vec16<T>::store(src, v);   // normalised / rotated (or, for text rows without norm, unchanged) values stay in qkv
      Vec16<T>::load(src, v);    // what reaches the buffer is exactly what qkv now holds
    }
    if (part == 1) {
      T *dst = kbuf + ((size_t)h * Lp + (row0 + i)) * dh + c;
      if (inplace) {
        Vec16<T>::store(dst, v);
      } else {
        *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<const uint4 *>(src);
      }
    }
    return;
  }
  // ---- V transpose tiles
  __shared__ T tile[64][64 + 2];
  const int bid = blockIdx.x - nbk;
  const int ctiles = (d + 63) / 64;
  const int r0 = (bid / ctiles) * 64, c0 = (bid % ctiles) * 64;
  for (int e = threadIdx.x; e < 64 * 64; e += 256) {
    int r = e >> 6, c = e & 63;
    if (r0 + r < rows && c0 + c < d) tile[r][c] = qkv[(size_t)(r0 + r) * ld + 2 * (size_t)d + c0 + c];
  }
  __syncthreads();
  for (int e = threadIdx.x; e < 64 * 64; e += 256) {
    int c = e >> 6, r = e & 63;
    if (r0 + r < rows && c0 + c < d) {
      int ch = c0 + c;
      int h = ch / dh, cc = ch % dh;
      vtbuf[((size_t)h * dh + cc) * Lp + row0 + r0 + r] = tile[r][c];
    }
  }
}

hipError_t launch_kv_scatter(const ScatterArgs &a, hipStream_t s) {
  if (a.rows <= 0) return hipSuccess;
  const int d = a.n_heads * a.head_dim;
  const int V = a.dt == DT_BF16 ? 8 : 4;
  int64_t kthreads = (int64_t)a.rows * ((a.rope || a.q_norm_w) ? 2 : 1) * (d / V);
  int nbk = (int)((kthreads + 255) / 256);
  int nbv = ((a.rows + 63) / 64) * ((d + 63) / 64);
  dim3 g(nbk + nbv);
  if (a.dt == DT_BF16)
    kv_scatter_kernel<bf16_t><<<g, 256, 0, s>>>((bf16_t *)a.qkv, a.ld, (bf16_t *)a.kbuf, (bf16_t *)a.vtbuf,
                                                a.rows_padded, a.n_heads, a.head_dim, a.row0, a.rows, a.rope,
                                                a.tok0, a.grid_w, a.theta, nbk, (const bf16_t *)a.q_norm_w,
                                                (const bf16_t *)a.k_norm_w, a.norm_eps, a.q_scale);
  else
    kv_scatter_kernel<float><<<g, 256, 0, s>>>((float *)a.qkv, a.ld, (float *)a.kbuf, (float *)a.vtbuf,
                                               a.rows_padded, a.n_heads, a.head_dim, a.row0, a.rows, a.rope, a.tok0,
                                               a.grid_w, a.theta, nbk, (const float *)a.q_norm_w, (const float *)a.k_norm_w,
                                               a.norm_eps, a.q_scale);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// split-KV combine: partial (unnormalised O, running max m, running sum l) per split -> normalised output.
// ws layout: O[splits][nq][H*dh] floats, then ml[splits][nq][H][2].
// ------------------------------------------------------------------------------------------------
size_t attention_ws_bytes(int nq, int n_heads, int head_dim, int splits) {
  if (splits <= 1) return 0;
  size_t o = (size_t)splits * nq * n_heads * head_dim;
  size_t ml = (size_t)splits * nq * n_heads * 2;
  return (o + ml) * sizeof(float);
}

// HALF: the partial outputs are normalised rows in fp16 (written by the direct-to-LDS bf16 attention kernel) instead of
// fp32 numerators; a split's weight then carries its denominator, and a thread takes eight channels (one 16-byte load per
// split) instead of four.
template <typename T, bool HALF = false, int G = 8>
__global__ __launch_bounds__(256) void attn_combine_kernel(const float *__restrict__ ws, T *__restrict__ out,
                                                           int64_t ldo, int nq, int H, int dh, int splits, int hpi) {
  // H counts heads over all images of the call (hpi per image); out rows are image-major
  constexpr int CH = HALF ? 8 : 4;
  const int d = H * dh;
  const int cpr = d / CH;
  int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (id >= (int64_t)nq * cpr) return;
  int i = (int)(id / cpr), ch = (int)(id % cpr) * CH;
  int h = ch / dh;
  const float *ml = ws + (size_t)splits * nq * d;
  // G splits at a time (eight, or four for launches of at most four splits, whose surplus slots would only repeat the
  // last split's loads), every load of the group issued before the first use: the loads of one thread are
  // independent, so a group costs one memory latency instead of one per split.  A split that saw no key (l <= 0) may
  // never have written its O rows: its values are dropped by selection, not by a zero weight.
  typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
  float M = -INFINITY, L = 0.f, o[CH];
#pragma unroll
  for (int t = 0; t < CH; ++t) o[t] = 0.f;
  for (int s0 = 0; s0 < splits; s0 += G) {
    float2 p[G];
    float v[G][CH];
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const int sidx = s0 + j < splits ? s0 + j : splits - 1;
      p[j] = *reinterpret_cast<const float2 *>(ml + (((size_t)sidx * nq + i) * H + h) * 2);
      if constexpr (HALF) {
        const f16x8 hv = *reinterpret_cast<const f16x8 *>(reinterpret_cast<const _Float16 *>(ws) + ((size_t)sidx * nq + i) * d + ch);
#pragma unroll
        for (int t = 0; t < CH; ++t) v[j][t] = (float)hv[t];
      } else {
        const float4 f = *reinterpret_cast<const float4 *>(ws + ((size_t)sidx * nq + i) * d + ch);
        v[j][0] = f.x; v[j][1] = f.y; v[j][2] = f.z; v[j][3] = f.w;
      }
    }
    float Mg = M;
#pragma unroll
    for (int j = 0; j < G; ++j)
      if (s0 + j < splits && p[j].y > 0.f) Mg = fmaxf(Mg, p[j].x);
    if (Mg == -INFINITY) continue;   // no key in this group or before it
    const float keep = expf(M - Mg);  // 0 for M = -inf
    L *= keep;
#pragma unroll
    for (int t = 0; t < CH; ++t) o[t] *= keep;
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const bool live = s0 + j < splits && p[j].y > 0.f;
      float wgt = live ? expf(p[j].x - Mg) : 0.f;
      if constexpr (HALF) {   // normalised rows: the weight carries the split's denominator
        wgt *= live ? p[j].y : 0.f;
        L += wgt;
      } else {
        L += live ? p[j].y * wgt : 0.f;
      }
#pragma unroll
      for (int t = 0; t < CH; ++t) o[t] += live ? v[j][t] * wgt : 0.f;
    }
    M = Mg;
  }
  float inv = 1.f / L;
  const int img = h / hpi;
  T *dst = out + ((size_t)img * nq + i) * ldo + (ch - img * hpi * dh);
#pragma unroll
  for (int t = 0; t < CH; ++t) Elem<T>::store(dst + t, o[t] * inv);
}

hipError_t launch_attn_combine(const AttnArgs &a, hipStream_t s) {
  const int B = a.batch > 1 ? a.batch : 1;
  const int d = a.n_heads * B * a.head_dim;
  const bool half = attn_partials_half(a);
  int64_t threads = (int64_t)a.nq * (d / (half ? 8 : 4));
  dim3 g((unsigned)((threads + 255) / 256));
  if (half && a.splits <= 4)
    attn_combine_kernel<bf16_t, true, 4><<<g, 256, 0, s>>>(a.ws, (bf16_t *)a.out, a.ldo, a.nq, a.n_heads * B, a.head_dim, a.splits, a.n_heads);
  else if (half)
    attn_combine_kernel<bf16_t, true><<<g, 256, 0, s>>>(a.ws, (bf16_t *)a.out, a.ldo, a.nq, a.n_heads * B, a.head_dim, a.splits, a.n_heads);
  else if (a.dt == DT_BF16)
    attn_combine_kernel<bf16_t><<<g, 256, 0, s>>>(a.ws, (bf16_t *)a.out, a.ldo, a.nq, a.n_heads * B, a.head_dim, a.splits, a.n_heads);
  else
    attn_combine_kernel<float><<<g, 256, 0, s>>>(a.ws, (float *)a.out, a.ldo, a.nq, a.n_heads * B, a.head_dim, a.splits, a.n_heads);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// RoPE (cos, sin) table of a call's rows: first half of a head's channel pairs <- grid row, second half <- grid column
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void rope_table_kernel(float2 *__restrict__ tab, int rows, int n_text, int tok0,
                                                         int grid_w, int dh, float theta) {
  const int half = dh >> 1, quarter = dh >> 2;
  int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (id >= (int64_t)rows * half) return;
  const int r = (int)(id / half), j = (int)(id % half);
  float cs = 1.f, sn = 0.f;
  if (r >= n_text) {
    const int tok = tok0 + (r - n_text);
    const int ia = j < quarter ? j : j - quarter;
    const float pos = j < quarter ? (float)(tok / grid_w) : (float)(tok % grid_w);
    const float freq = exp2f(-log2f(theta) * (4.0f * (float)ia / (float)dh));
    sincosf(pos * freq, &sn, &cs);
  }
  tab[id] = make_float2(cs, sn);
}

hipError_t launch_rope_table(void *tab, int rows, int n_text, int tok0, int grid_w, int dh, float theta, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  int64_t n = (int64_t)rows * (dh >> 1);
  rope_table_kernel<<<dim3((unsigned)((n + 255) / 256)), 256, 0, s>>>((float2 *)tab, rows, n_text, tok0, grid_w, dh, theta);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// out = a * x + b * y: the element-wise sampler update between diffusion steps (Sec. 2, Eq. 1): a = 1 is the Euler /
// flow form x + dt * eps, general (a, b) covers the deterministic DDIM-type rules that are linear in x_t and eps
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void axpby_kernel(const float *__restrict__ x, const float *__restrict__ y, float a,
                                                    float b, float *__restrict__ out, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * 256;
  if (a == 1.0f) {
    for (; i < n; i += stride) out[i] = fmaf(b, y[i], x[i]);
  } else {
    for (; i < n; i += stride) out[i] = fmaf(b, y[i], a * x[i]);
  }
}

hipError_t launch_axpby(const float *x, const float *y, float a, float b, float *out, int64_t n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  axpby_kernel<<<dim3((unsigned)blocks), 256, 0, s>>>(x, y, a, b, out, n);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void fill_zero_kernel(uint4 *p, size_t n16) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  size_t stride = (size_t)gridDim.x * 256;
  for (; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}

hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  size_t n16 = bytes / 16;
  unsigned blocks = (unsigned)((n16 + 255) / 256);
  if (blocks > 8192) blocks = 8192;
  fill_zero_kernel<<<dim3(blocks), 256, 0, s>>>((uint4 *)p, n16);
  return hipGetLastError();
}

}  // namespace pf
