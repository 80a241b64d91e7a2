// bf16 MFMA GEMM for gfx950: C = epilogue(A W^T + bias), A [M,K] and W [N,K] both contiguous along K,
// fp32 accumulation in v_mfma_f32_32x32x16_bf16.  256 threads = 4 wavefronts in a 2x2 arrangement; the
// block tile BM x BN x 64 is staged through LDS with a register prefetch of the next K tile
// (two LDS buffers, one barrier per K tile).
#include "common.h"
#include "epilogue.h"
#include "ops.h"

namespace pf {

namespace {

constexpr int BK = 64;        // K elements per LDS stage
constexpr int LDS_LD = BK + 8;  // padded row stride (elements): 144 B, conflict-free 16-byte reads

template <int BM, int BN>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(const bf16_t *__restrict__ A, int64_t lda,
                                                        const bf16_t *__restrict__ W, int64_t ldw, int M, int N, int K,
                                                        Epilogue<bf16_t> epi) {
  constexpr int WM = BM / 2, WN = BN / 2;  // wave tile
  constexpr int MI = WM / 32, NI = WN / 32;
  constexpr int A_CHUNKS = BM * (BK / 8) / 256;  // 16-byte chunks staged per thread
  constexpr int W_CHUNKS = BN * (BK / 8) / 256;
  static_assert(A_CHUNKS >= 1 && W_CHUNKS >= 1, "tile too small for 256 threads");

  __shared__ __attribute__((aligned(16))) bf16_t As[2][BM * LDS_LD];
  __shared__ __attribute__((aligned(16))) bf16_t Ws[2][BN * LDS_LD];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;

  f32x16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  uint4 ra[A_CHUNKS], rw[W_CHUNKS];
  auto gload = [&](int k0) {
#pragma unroll
    for (int u = 0; u < A_CHUNKS; ++u) {
      int id = tid + 256 * u;
      int r = id >> 3, kc = (id & 7) * 8;
      ra[u] = make_uint4(0, 0, 0, 0);
      if (m0 + r < M && k0 + kc < K) ra[u] = *reinterpret_cast<const uint4 *>(A + (size_t)(m0 + r) * lda + k0 + kc);
    }
#pragma unroll
    for (int u = 0; u < W_CHUNKS; ++u) {
      int id = tid + 256 * u;
      int r = id >> 3, kc = (id & 7) * 8;
      rw[u] = make_uint4(0, 0, 0, 0);
      if (n0 + r < N && k0 + kc < K) rw[u] = *reinterpret_cast<const uint4 *>(W + (size_t)(n0 + r) * ldw + k0 + kc);
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int u = 0; u < A_CHUNKS; ++u) {
      int id = tid + 256 * u;
      int r = id >> 3, kc = (id & 7) * 8;
      *reinterpret_cast<uint4 *>(&As[buf][r * LDS_LD + kc]) = ra[u];
    }
#pragma unroll
    for (int u = 0; u < W_CHUNKS; ++u) {
      int id = tid + 256 * u;
      int r = id >> 3, kc = (id & 7) * 8;
      *reinterpret_cast<uint4 *>(&Ws[buf][r * LDS_LD + kc]) = rw[u];
    }
  };

  const int nk = (K + BK - 1) / BK;
  gload(0);
  sstore(0);
  __syncthreads();
  const int frow = lane & 31, fk = (lane >> 5) * 8;
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) gload((kt + 1) * BK);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 af[MI], wf[NI];
#pragma unroll
      for (int i = 0; i < MI; ++i)
        af[i] = *reinterpret_cast<const bf16x8 *>(&As[buf][(wm * WM + i * 32 + frow) * LDS_LD + ks * 16 + fk]);
#pragma unroll
      for (int j = 0; j < NI; ++j)
        wf[j] = *reinterpret_cast<const bf16x8 *>(&Ws[buf][(wn * WN + j * 32 + frow) * LDS_LD + ks * 16 + fk]);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], wf[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) sstore(buf ^ 1);
    __syncthreads();
  }

  // accumulator layout of a 32x32 block: lane -> column (lane & 31); register r -> row 8*(r/4) + 4*(lane/32) + r%4
#pragma unroll
  for (int j = 0; j < NI; ++j) {
    int col = n0 + wn * WN + j * 32 + (lane & 31);
    if (col >= N) continue;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        int row = m0 + wm * WM + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row < M) epi.apply(row, col, acc[i][j][r]);
      }
    }
  }
}

template <int BM, int BN>
void launch_tile(const GemmArgs &a, hipStream_t s) {
  dim3 g((a.N + BN - 1) / BN, (a.M + BM - 1) / BM);
  gemm_mfma_kernel<BM, BN><<<g, 256, 0, s>>>((const bf16_t *)a.A, a.lda, (const bf16_t *)a.W, a.ldw, a.M, a.N, a.K,
                                             make_epilogue<bf16_t>(a));
}

}  // namespace

hipError_t launch_gemm_mfma(const GemmArgs &a, hipStream_t s) {
  if (a.M <= 0 || a.N <= 0) return hipSuccess;
  auto tiles = [&](int bm, int bn) { return (int64_t)((a.M + bm - 1) / bm) * ((a.N + bn - 1) / bn); };
  // Largest tile that still gives every CU (256) roughly two workgroups; otherwise the smallest.
  if (tiles(128, 128) >= 512) launch_tile<128, 128>(a, s);
  else if (tiles(64, 128) >= 384) launch_tile<64, 128>(a, s);
  else launch_tile<64, 64>(a, s);
  return hipGetLastError();
}

}  // namespace pf
