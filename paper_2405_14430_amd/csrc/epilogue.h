// GEMM epilogues shared by the SIMT and MFMA GEMM kernels.
//   mode 0: C[row][col] (dtype) = acc + bias[col], GELU on columns >= gelu_from
//   mode 1: X[row][col] (fp32)  = R[row][col] + gate[col] * (acc + bias[col]); optional rounded copy in C2
// A mode-0 launch that is a QKV projection may carry a KvRoute: its k and v columns then go straight into a layer's
// K / V^T buffers at the patch's rows (the write-before-attend step of PipeFusion Sec. 3.3) instead of into C, and
// q and k are rotated with a precomputed (cos, sin) table when the stage uses RoPE.  Only the vectorised LDS-staged
// epilogue of the direct-to-LDS GEMM kernels implements the route.
#pragma once
#include "common.h"

namespace pf {

// N = 3d columns: [0,d) q -> C, [d,2d) k -> kbuf[h][brow][c], [2d,3d) v -> vtbuf[h][c][brow].
// GEMM row r maps to buffer row (r < split ? row0a + r : row0b + r - split): text rows first, then the image patch.
struct KvRoute {
  void *kbuf, *vtbuf;          // nullptr kbuf: no routing
  int Lp, dh, d;
  int split, row0a, row0b;
  const float2 *rope;          // [rows of one image][dh/2] (cos, sin) per GEMM row, or nullptr
  int seg;                     // > 0: GEMM rows are image-major, seg rows per image; mapping applies inside the image
  int64_t img_stride;          // elements between consecutive images' K (and V^T) buffers
  float q_scale;               // != 0: q columns are multiplied by it (the attention kernel's log2(e) / sqrt(dh))
};

template <typename T>
struct Epilogue {
  KvRoute kv;
  const T *bias;
  void *C; int64_t ldc;
  int mode, gelu_from, gelu_tanh;
  const float *gate;
  int gate_seg; int64_t gate_stride;   // gate_seg > 0: row r reads gate + (r / gate_seg) * gate_stride
  const float *R; int64_t ldr;
  T *C2; int64_t ldc2;

  __device__ __forceinline__ const float *gate_of(int row) const {
    return gate_seg > 0 ? gate + (int64_t)(row / gate_seg) * gate_stride : gate;
  }

  __device__ __forceinline__ void apply(int row, int col, float acc) const {
    float v = acc + (bias ? to_f32(bias[col]) : 0.f);
    if (mode == 0) {
      if (col >= gelu_from) v = gelu_f(v, gelu_tanh);
      Elem<T>::store(reinterpret_cast<T *>(C) + (size_t)row * ldc + col, v);
    } else {
      float g = gate ? gate_of(row)[col] : 1.f;
      float x = R[(size_t)row * ldr + col] + g * v;
      reinterpret_cast<float *>(C)[(size_t)row * ldc + col] = x;
      if (C2) Elem<T>::store(C2 + (size_t)row * ldc2 + col, x);
    }
  }
};

template <typename T, typename Args>
inline Epilogue<T> make_epilogue(const Args &a) {
  Epilogue<T> e;
  e.kv = KvRoute{a.kvr.kbuf, a.kvr.vtbuf, a.kvr.Lp, a.kvr.dh, a.kvr.d, a.kvr.split, a.kvr.row0a, a.kvr.row0b,
                 (const float2 *)a.kvr.rope, a.kvr.seg, a.kvr.img_stride, a.kvr.q_scale};
  e.bias = (const T *)a.bias; e.C = a.C; e.ldc = a.ldc; e.mode = a.epilogue; e.gelu_from = a.gelu_from;
  e.gelu_tanh = a.gelu_tanh; e.gate = a.gate; e.gate_seg = a.gate_seg; e.gate_stride = a.gate_stride; e.R = a.R; e.ldr = a.ldr; e.C2 = (T *)a.C2; e.ldc2 = a.ldc2;
  return e;
}

}  // namespace pf
