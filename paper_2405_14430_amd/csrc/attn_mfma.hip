// Flash-style patch attention for gfx950 (bf16 operands, fp32 accumulation and softmax statistics).
//
// The patch's queries attend over ALL rows of the layer's K/V buffer, fresh and stale alike (PipeFusion
// Sec. 3.3).  Per workgroup: 128 queries of one head (4 wavefronts x 32 queries) and one split of the key
// range; K tiles [64][dh] and V^T tiles [dh][64] are staged in LDS (register prefetch, two buffers).
//
// Everything is computed transposed so that a lane owns one query column:
//   S^T[kv][q] = K[kv][:] . Q[q][:]        A = K tile (LDS), B = Q fragments (registers)
//   O^T[c][q] += V^T[c][kv] . P^T[kv][q]   A = V^T tile (LDS), B = P^T, taken straight from the S^T accumulator
// In the 32x32 accumulator layout lane l holds column l%32 and rows 8*(r/4) + 4*(l/32) + r%4, so the online-softmax
// maximum / sum are in-lane reductions plus one exchange with lane l^32, the rescale of O^T is per lane, and the
// eight accumulator registers 8s..8s+7 are exactly one K=16 B-operand (the matching A-operand gathers the same
// kv rows from the V^T tile with two 8-byte LDS reads).
#include "common.h"
#include "ops.h"

namespace pf {

namespace {

constexpr int TQ = 128;  // queries per workgroup
constexpr int TK = 64;   // kv rows per LDS tile
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <int DH>
struct AttnCfg {
  static constexpr int KS16 = DH / 16;                 // full K=16 steps of the QK^T contraction
  static constexpr bool TAIL8 = (DH % 16) == 8;        // one extra K=8 step (dh = 72)
  static constexpr int KLD = TAIL8 ? DH : DH + 8;      // LDS row stride of the K tile (elements)
  static constexpr int CB = (DH + 31) / 32;            // 32-row blocks of O^T
  static constexpr int VROWS = CB * 32;
  static constexpr int VLD = TK + 4;                   // LDS row stride of the V^T tile (elements)
  static constexpr int K_ELEMS = TK * KLD;
  static constexpr int V_ELEMS = VROWS * VLD;
  static constexpr int KCH = (TK * (DH / 8) + 255) / 256;  // 16-byte chunks per thread, K tile
  static constexpr int VCH = (DH * (TK / 8) + 255) / 256;  // V^T tile
};

template <int DH>
__global__ __launch_bounds__(256) void attn_mfma_kernel(const bf16_t *__restrict__ q, int64_t ldq,
                                                        const bf16_t *__restrict__ kbuf,
                                                        const bf16_t *__restrict__ vtbuf, int kv_rows, int Lp, int H,
                                                        int dh, bf16_t *__restrict__ out, int64_t ldo, int nq,
                                                        int splits, float *__restrict__ ws, int hpi) {
  // H counts heads over all images of the call (hpi per image); q / out rows are image-major
  using C = AttnCfg<DH>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t *Ks = reinterpret_cast<bf16_t *>(smem_raw);            // [2][K_ELEMS]
  bf16_t *Vs = Ks + 2 * C::K_ELEMS;                             // [2][V_ELEMS]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hi = lane >> 5;
  const int h = blockIdx.y, sp = blockIdx.z;
  const int q0 = blockIdx.x * TQ + wave * 32;
  const int dh8 = dh >> 3;

  // zero LDS once: padding columns / rows are never written by the tile loads
  for (int e = tid; e < (2 * C::K_ELEMS + 2 * C::V_ELEMS) / 8; e += 256)
    reinterpret_cast<uint4 *>(smem_raw)[e] = make_uint4(0, 0, 0, 0);

  // split of the key range, in whole tiles
  const int tiles = (kv_rows + TK - 1) / TK;
  const int tps = (tiles + splits - 1) / splits;
  const int t_begin = sp * tps, t_end = min(tiles, (sp + 1) * tps);
  const bf16_t *kh = kbuf + (size_t)h * Lp * dh;
  const bf16_t *vh = vtbuf + (size_t)h * dh * Lp;

  // Q fragments (B operand): lane holds query q0 + l32, channels ks*16 + 8*hi .. +7
  bf16x8 qf[C::KS16];
  bf16x4 qt = {0, 0, 0, 0};
  {
    const int qi = q0 + l32;
    const bf16_t *qp = q + ((size_t)(h / hpi) * nq + qi) * ldq + (size_t)(h % hpi) * dh;
#pragma unroll
    for (int ks = 0; ks < C::KS16; ++ks) {
      int c = ks * 16 + hi * 8;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (qi < nq && c < dh) v = *reinterpret_cast<const uint4 *>(qp + c);
      qf[ks] = __builtin_bit_cast(bf16x8, v);
    }
    if constexpr (C::TAIL8) {
      int c = C::KS16 * 16 + hi * 4;
      uint2 v = make_uint2(0, 0);
      if (qi < nq && c < dh) v = *reinterpret_cast<const uint2 *>(qp + c);
      qt = __builtin_bit_cast(bf16x4, v);
    }
  }

  uint4 rk[C::KCH], rv[C::VCH];
  auto gload = [&](int t) {
    const int j0 = t * TK;
#pragma unroll
    for (int u = 0; u < C::KCH; ++u) {
      int id = tid + 256 * u;
      int r = id / dh8, c = (id % dh8) * 8;
      rk[u] = make_uint4(0, 0, 0, 0);
      if (r < TK) rk[u] = *reinterpret_cast<const uint4 *>(kh + (size_t)(j0 + r) * dh + c);
    }
#pragma unroll
    for (int u = 0; u < C::VCH; ++u) {
      int id = tid + 256 * u;
      int c = id >> 3, k8 = (id & 7) * 8;
      rv[u] = make_uint4(0, 0, 0, 0);
      if (c < dh) rv[u] = *reinterpret_cast<const uint4 *>(vh + (size_t)c * Lp + j0 + k8);
    }
  };
  auto sstore = [&](int buf) {
    bf16_t *kd = Ks + buf * C::K_ELEMS;
    bf16_t *vd = Vs + buf * C::V_ELEMS;
#pragma unroll
    for (int u = 0; u < C::KCH; ++u) {
      int id = tid + 256 * u;
      int r = id / dh8, c = (id % dh8) * 8;
      if (r < TK) *reinterpret_cast<uint4 *>(kd + r * C::KLD + c) = rk[u];
    }
#pragma unroll
    for (int u = 0; u < C::VCH; ++u) {
      int id = tid + 256 * u;
      int c = id >> 3, k8 = (id & 7) * 8;
      if (c < dh) {  // row stride 136 B: only 8-byte aligned
        uint2 *p = reinterpret_cast<uint2 *>(vd + c * C::VLD + k8);
        p[0] = make_uint2(rv[u].x, rv[u].y);
        p[1] = make_uint2(rv[u].z, rv[u].w);
      }
    }
  };

  f32x16 oacc[C::CB];
#pragma unroll
  for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[cb][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;   // log2 domain maximum; per-lane partial sum
  const float sl2 = kLog2e / sqrtf((float)dh);

  __syncthreads();  // LDS zero fill done
  if (t_begin < t_end) {
    gload(t_begin);
    sstore(0);
  }
  __syncthreads();

  for (int t = t_begin; t < t_end; ++t) {
    const int buf = (t - t_begin) & 1;
    if (t + 1 < t_end) gload(t + 1);
    const bf16_t *kt = Ks + buf * C::K_ELEMS;
    const bf16_t *vt = Vs + buf * C::V_ELEMS;

    // ---- S^T = K . Q^T for the two 32-row blocks of the tile
    f32x16 sacc[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[b][r] = 0.f;
      const bf16_t *krow = kt + (b * 32 + l32) * C::KLD;
#pragma unroll
      for (int ks = 0; ks < C::KS16; ++ks) {
        bf16x8 kf = *reinterpret_cast<const bf16x8 *>(krow + ks * 16 + hi * 8);
        sacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], sacc[b], 0, 0, 0);
      }
      if constexpr (C::TAIL8) {
        bf16x4 kf4 = *reinterpret_cast<const bf16x4 *>(krow + C::KS16 * 16 + hi * 4);
        sacc[b] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(__builtin_bit_cast(short4v, kf4),
                                                           __builtin_bit_cast(short4v, qt), sacc[b], 0, 0, 0);
      }
    }
    // ---- scale to the log2 domain, mask the ragged end, online softmax
    const int jbase = t * TK + 4 * hi;
    const bool ragged = (t + 1) * TK > kv_rows;
    float tmax = -INFINITY;
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float v = sacc[b][r] * sl2;
        if (ragged) {
          int j = jbase + b * 32 + 8 * (r >> 2) + (r & 3);
          if (j >= kv_rows) v = -INFINITY;
        }
        sacc[b][r] = v;
        tmax = fmaxf(tmax, v);
      }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave));
    const float m_new = fmaxf(m_run, tmax);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    float psum = 0.f;
    bf16x8 pf[2][2];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float p = __builtin_amdgcn_exp2f(sacc[b][r] - m_new);
        bf16_t pb = (bf16_t)p;
        psum += (float)pb;   // the sum uses the rounded weights that multiply V
        pf[b][r >> 3][r & 7] = pb;
      }
    l_run = l_run * alpha + psum;
#pragma unroll
    for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[cb][r] *= alpha;
    // ---- O^T += V^T . P^T
#pragma unroll
    for (int cb = 0; cb < C::CB; ++cb) {
      const bf16_t *vrow = vt + (cb * 32 + l32) * C::VLD + 4 * hi;
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const bf16_t *vp = vrow + b * 32 + s2 * 16;
          uint2 lo = *reinterpret_cast<const uint2 *>(vp);
          uint2 hi2 = *reinterpret_cast<const uint2 *>(vp + 8);
          uint4 both = make_uint4(lo.x, lo.y, hi2.x, hi2.y);
          oacc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pf[b][s2], oacc[cb], 0, 0, 0);
        }
    }
    if (t + 1 < t_end) sstore(buf ^ 1);
    __syncthreads();
  }

  // ---- finish: combine the two half-lane partial sums, normalise or emit partials
  const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
  const int qi = q0 + l32;
  if (qi >= nq) return;
  const int d = H * dh;
  if (splits == 1) {
    const float inv = 1.f / l_tot;
    bf16_t *op = out + ((size_t)(h / hpi) * nq + qi) * ldo + (size_t)(h % hpi) * dh;
#pragma unroll
    for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        int c = cb * 32 + 8 * g + 4 * hi;
        if (c < dh) {
          bf16x4 o4;
#pragma unroll
          for (int e = 0; e < 4; ++e) o4[e] = (bf16_t)(oacc[cb][4 * g + e] * inv);
          *reinterpret_cast<bf16x4 *>(op + c) = o4;
        }
      }
  } else {
    float *op = ws + ((size_t)sp * nq + qi) * d + (size_t)h * dh;
#pragma unroll
    for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        int c = cb * 32 + 8 * g + 4 * hi;
        if (c < dh)
          *reinterpret_cast<float4 *>(op + c) =
              make_float4(oacc[cb][4 * g], oacc[cb][4 * g + 1], oacc[cb][4 * g + 2], oacc[cb][4 * g + 3]);
      }
    if (hi == 0) {
      float *ml = ws + (size_t)splits * nq * d + (((size_t)sp * nq + qi) * H + h) * 2;
      ml[0] = m_run * kLn2;   // natural-log domain for the combine kernel
      ml[1] = l_tot;
    }
  }
}

template <int DH>
hipError_t attn_launch(const AttnArgs &a, hipStream_t s) {
  using C = AttnCfg<DH>;
  const int B = a.batch > 1 ? a.batch : 1;
  dim3 g((a.nq + TQ - 1) / TQ, a.n_heads * B, a.splits);
  constexpr int smem = (2 * C::K_ELEMS + 2 * C::V_ELEMS) * (int)sizeof(bf16_t);
  if (hipError_t e = allow_dynamic_lds<&attn_mfma_kernel<DH>, smem>(); e != hipSuccess) return e;
  attn_mfma_kernel<DH><<<g, 256, smem, s>>>((const bf16_t *)a.q, a.ldq, (const bf16_t *)a.kbuf,
                                            (const bf16_t *)a.vtbuf, a.kv_rows, a.rows_padded, a.n_heads * B, a.head_dim,
                                            (bf16_t *)a.out, a.ldo, a.nq, a.splits, a.ws, a.n_heads);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_mfma(const AttnArgs &a, hipStream_t s) {
  if (a.nq <= 0) return hipSuccess;
  const int dh = a.head_dim;
  if (dh <= 64) return attn_launch<64>(a, s);
  if (dh <= 72) return attn_launch<72>(a, s);
  if (dh <= 96) return attn_launch<96>(a, s);
  return attn_launch<128>(a, s);
}

}  // namespace pf
