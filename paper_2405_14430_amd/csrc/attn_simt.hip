// Plain SIMT attention of patch queries over a full-sequence K/V buffer (PipeFusion Sec. 3.3: the buffer
// mixes fresh and stale rows; the kernel does not care which is which).  One query row per thread, one
// wavefront per workgroup, K/V streamed through LDS in tiles of 32 rows, online softmax per thread.
// Used for the fp32 dtype and as the forced-SIMT path for bf16.
#include "common.h"
#include "ops.h"

namespace pf {

// K [H][Lp][dh], V^T [H][dh][Lp].  DH >= dh is the compile-time register width.
template <typename T, int DH>
__global__ __launch_bounds__(64) void attn_simt_kernel(const T *__restrict__ q, int64_t ldq, const T *__restrict__ kbuf,
                                                       const T *__restrict__ vtbuf, int kv_rows, int Lp, int H, int dh,
                                                       T *__restrict__ out, int64_t ldo, int nq, int splits,
                                                       float *__restrict__ ws, int hpi) {
  // H counts heads over all images of the call (hpi per image); q / out rows are image-major
  constexpr int TK = 32;
  __shared__ __attribute__((aligned(16))) float Ks[TK][DH];
  __shared__ __attribute__((aligned(16))) float Vs[DH][TK];
  const int lane = threadIdx.x;
  const int h = blockIdx.y, sp = blockIdx.z;
  const int i = blockIdx.x * 64 + lane;
  const bool active = i < nq;
  const float sm_scale = 1.0f / sqrtf((float)dh);

  float qr[DH], o[DH];
#pragma unroll
  for (int c = 0; c < DH; ++c) {
    qr[c] = (active && c < dh) ? to_f32(q[((size_t)(h / hpi) * nq + i) * ldq + (size_t)(h % hpi) * dh + c]) * sm_scale : 0.f;
    o[c] = 0.f;
  }
  float m = -INFINITY, l = 0.f;

  const int tiles = (kv_rows + TK - 1) / TK;
  const int tps = (tiles + splits - 1) / splits;
  const int j_begin = sp * tps * TK;
  const int j_end = min(kv_rows, (sp + 1) * tps * TK);
  const T *kh = kbuf + (size_t)h * Lp * dh;
  const T *vh = vtbuf + (size_t)h * dh * Lp;

  for (int j0 = j_begin; j0 < j_end; j0 += TK) {
    __syncthreads();
    for (int e = lane; e < TK * DH; e += 64) {
      int r = e / DH, c = e % DH;
      Ks[r][c] = (j0 + r < j_end && c < dh) ? to_f32(kh[(size_t)(j0 + r) * dh + c]) : 0.f;
    }
    for (int e = lane; e < DH * TK; e += 64) {
      int c = e / TK, r = e % TK;
      Vs[c][r] = (j0 + r < j_end && c < dh) ? to_f32(vh[(size_t)c * Lp + j0 + r]) : 0.f;
    }
    __syncthreads();
    float sc[TK];
    float tmax = -INFINITY;
#pragma unroll
    for (int r = 0; r < TK; ++r) {
      float acc = 0.f;
#pragma unroll
      for (int c = 0; c < DH; c += 4) {
        float4 kv = *reinterpret_cast<const float4 *>(&Ks[r][c]);
        acc = fmaf(qr[c], kv.x, acc);
        acc = fmaf(qr[c + 1], kv.y, acc);
        acc = fmaf(qr[c + 2], kv.z, acc);
        acc = fmaf(qr[c + 3], kv.w, acc);
      }
      sc[r] = (j0 + r < j_end) ? acc : -INFINITY;
      tmax = fmaxf(tmax, sc[r]);
    }
    float m_new = fmaxf(m, tmax);
    float alpha = expf(m - m_new);  // m = -inf on the first tile: exp(-inf) = 0
    float psum = 0.f;
#pragma unroll
    for (int r = 0; r < TK; ++r) {
      sc[r] = expf(sc[r] - m_new);
      psum += sc[r];
    }
    l = l * alpha + psum;
    m = m_new;
#pragma unroll
    for (int c = 0; c < DH; ++c) {
      float acc = o[c] * alpha;
#pragma unroll
      for (int r = 0; r < TK; r += 4) {
        float4 vv = *reinterpret_cast<const float4 *>(&Vs[c][r]);
        acc = fmaf(sc[r], vv.x, acc);
        acc = fmaf(sc[r + 1], vv.y, acc);
        acc = fmaf(sc[r + 2], vv.z, acc);
        acc = fmaf(sc[r + 3], vv.w, acc);
      }
      o[c] = acc;
    }
  }
  if (!active) return;
  const int d = H * dh;
  if (splits == 1) {
    float inv = 1.f / l;
#pragma unroll
    for (int c = 0; c < DH; ++c)
      if (c < dh) Elem<T>::store(out + ((size_t)(h / hpi) * nq + i) * ldo + (size_t)(h % hpi) * dh + c, o[c] * inv);
  } else {
    float *op = ws + ((size_t)sp * nq + i) * d + (size_t)h * dh;
#pragma unroll
    for (int c = 0; c < DH; ++c)
      if (c < dh) op[c] = o[c];
    float *ml = ws + (size_t)splits * nq * d + (((size_t)sp * nq + i) * H + h) * 2;
    ml[0] = m;
    ml[1] = l;
  }
}

template <typename T>
static hipError_t attn_simt_dispatch(const AttnArgs &a, hipStream_t s) {
  const int B = a.batch > 1 ? a.batch : 1;
  dim3 g((a.nq + 63) / 64, a.n_heads * B, a.splits);
#define PF_ATTN_SIMT(DH)                                                                                              \
  attn_simt_kernel<T, DH><<<g, 64, 0, s>>>((const T *)a.q, a.ldq, (const T *)a.kbuf, (const T *)a.vtbuf, a.kv_rows,     \
                                           a.rows_padded, a.n_heads * B, a.head_dim, (T *)a.out, a.ldo, a.nq, a.splits, \
                                           a.ws, a.n_heads)
  if (a.head_dim <= 64) PF_ATTN_SIMT(64);
  else if (a.head_dim <= 72) PF_ATTN_SIMT(72);
  else PF_ATTN_SIMT(128);
#undef PF_ATTN_SIMT
  return hipGetLastError();
}

hipError_t launch_attn_simt(const AttnArgs &a, hipStream_t s) {
  if (a.nq <= 0) return hipSuccess;
  return a.dt == DT_BF16 ? attn_simt_dispatch<bf16_t>(a, s) : attn_simt_dispatch<float>(a, s);
}

}  // namespace pf
