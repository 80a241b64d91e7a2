// Plain LDS-tiled SIMT GEMM, C = epilogue(A W^T + bias), fp32 accumulation.  Used for the fp32 dtype and as
// the forced-SIMT path for bf16.  64x64 output tile per 256-thread workgroup, 4x4 outputs per thread.
#include "common.h"
#include "epilogue.h"
#include "ops.h"

namespace pf {

template <typename T>
__global__ __launch_bounds__(256) void gemm_simt_kernel(const T *__restrict__ A, int64_t lda, const T *__restrict__ W,
                                                        int64_t ldw, int M, int N, int K, Epilogue<T> epi) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float As[BK][BM + 4];
  __shared__ float Ws[BK][BN + 4];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int lr = tid >> 2, lk = (tid & 3) * 4;  // this thread stages row lr, k offsets lk..lk+3 of both tiles
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += BK) {
    float a[4] = {0.f, 0.f, 0.f, 0.f}, w[4] = {0.f, 0.f, 0.f, 0.f};
    if (k0 + lk < K) {
      if (m0 + lr < M) {
        const T *p = A + (size_t)(m0 + lr) * lda + k0 + lk;
#pragma unroll
        for (int t = 0; t < 4; ++t) a[t] = to_f32(p[t]);
      }
      if (n0 + lr < N) {
        const T *p = W + (size_t)(n0 + lr) * ldw + k0 + lk;
#pragma unroll
        for (int t = 0; t < 4; ++t) w[t] = to_f32(p[t]);
      }
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      As[lk + t][lr] = a[t];
      Ws[lk + t][lr] = w[t];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < BK; ++k) {
      float4 av = *reinterpret_cast<const float4 *>(&As[k][ty * 4]);
      float4 wv = *reinterpret_cast<const float4 *>(&Ws[k][tx * 4]);
      float ar[4] = {av.x, av.y, av.z, av.w}, wr[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(ar[i], wr[j], acc[i][j]);
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int row = m0 + ty * 4 + i;
    if (row >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int col = n0 + tx * 4 + j;
      if (col < N) epi.apply(row, col, acc[i][j]);
    }
  }
}

hipError_t launch_gemm_simt(const GemmArgs &a, hipStream_t s) {
  if (a.M <= 0 || a.N <= 0) return hipSuccess;
  dim3 g((a.N + 63) / 64, (a.M + 63) / 64);
  if (a.dt == DT_BF16)
    gemm_simt_kernel<bf16_t><<<g, 256, 0, s>>>((const bf16_t *)a.A, a.lda, (const bf16_t *)a.W, a.ldw, a.M, a.N, a.K,
                                               make_epilogue<bf16_t>(a));
  else
    gemm_simt_kernel<float><<<g, 256, 0, s>>>((const float *)a.A, a.lda, (const float *)a.W, a.ldw, a.M, a.N, a.K,
                                              make_epilogue<float>(a));
  return hipGetLastError();
}

}  // namespace pf
