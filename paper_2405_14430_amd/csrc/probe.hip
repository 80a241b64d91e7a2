// Measurement aid: what the matrix pipes of this chip sustain when nothing else competes for them.
// A register-only loop of v_mfma_f32_32x32x16_bf16 (two independent accumulators per wave, two waves per SIMD on every
// CU); the benchmark times it next to the stage so that kernel rates can be read against a measured ceiling at the clock
// the chip actually holds under a matrix load, not only against the data-sheet figure.
#include "common.h"
#include "ops.h"

namespace pf {

namespace {
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8p __attribute__((ext_vector_type(8)));

__global__ __launch_bounds__(256, 2) void mfma_loop_kernel(float *__restrict__ out, int iters) {
  const int lane = threadIdx.x & 63;
  bf16x8p a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(0.001f * lane + 0.01f * i);
    b[i] = (__bf16)(0.01f * i);
  }
  f32x16 acc0 = {0}, acc1 = {0};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < 16; ++m) {
      acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, acc1, 0, 0, 0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += acc0[i] + acc1[i];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}
}  // namespace

// flops of one launch: workgroups * 4 waves * iters * 32 MFMAs * 2*32*32*16
hipError_t launch_mfma_loop(float *out, int workgroups, int iters, hipStream_t s) {
  mfma_loop_kernel<<<dim3((unsigned)workgroups), 256, 0, s>>>(out, iters);
  return hipGetLastError();
}

}  // namespace pf
