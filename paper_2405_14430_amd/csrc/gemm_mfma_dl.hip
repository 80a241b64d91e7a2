// bf16 MFMA GEMMs with direct global->LDS loads (gfx950): C = epilogue(A W^T + bias), A [M,K], W [N,K], both
// contiguous along K, K a multiple of 64.
//
// Tiles are brought in with global_load_lds_dwordx4: one instruction moves 64 x 16 B = 1 KB = eight 128-byte tile
// rows (64 bf16 of K each), lane l filling row l/8, 16-byte slot l%8.  The LDS side of such a load is lane-linear (no
// padding possible), so bank conflicts are avoided with an XOR swizzle: chunk c (8 bf16) of tile row r is kept in slot
// c ^ ((r >> 1) & 7); the loading lane picks its global chunk accordingly and the MFMA fragment reads undo it.  Rows
// beyond M (or N) are clamped to the last valid row: they only feed accumulators that the epilogue never stores.
//
// Two kernels share that machinery:
//  * gemm_tile_kernel<BM,BN,NSTAGE>: 2x2 wavefronts share one BM x BN tile; NSTAGE LDS stages, one s_barrier per K
//    tile.  For GEMMs with enough tiles to fill the chip.
//  * gemm_wavek_kernel<BM,BN>: for skinny GEMMs (n = 512 patch rows: a few hundred tiles at most).  The four
//    wavefronts of a workgroup split K between them: each streams its own K tiles through a private two-stage LDS
//    ring with no workgroup barrier in the loop, which quadruples the loads in flight per CU and divides the serial
//    chain of K iterations by four; the four partial tiles are then summed through LDS.
// Both finish through LDS: the fp32 tile is laid out row-major and every thread applies the epilogue to runs of 8
// consecutive columns (16-byte bf16 stores, 32-byte fp32 stores).
#include <mutex>
#include <type_traits>

#include "common.h"
#include "epilogue.h"
#include "ops.h"

namespace pf {

namespace {

constexpr int BK = 64;
constexpr int ROW_BYTES = BK * 2;  // 128

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// s_waitcnt vmcnt(behind * LPS) for a wave-uniform run-time `behind` in [0, MAXB] (the count is an immediate)
template <int LPS, int MAXB>
__device__ __forceinline__ void wait_tiles_behind(int behind) {
  static_assert(MAXB * LPS <= 63, "vmcnt is a 6-bit counter");
  if constexpr (MAXB <= 0) {
    wait_vmcnt<0>();
  } else {
    if (behind >= MAXB) wait_vmcnt<MAXB * LPS>();
    else wait_tiles_behind<LPS, MAXB - 1>(behind);
  }
}

// Tile loads are raw-buffer loads into LDS: a wave-uniform resource over the rows of the operand that the tile starts
// at, a wave-uniform byte offset (the K position) and one 32-bit per-lane byte offset.  Against global loads with a
// 64-bit address per lane that saves the 64-bit address arithmetic and half the address registers of every load
// (same-box A/B inside the stages: Flux-scale QKV 141 -> 136 us, MLP-up 173 -> 165 us, long-sequence PixArt QKV 60 ->
// 53 us).  The resource spans 2 GB from its base and the offsets are built from row indices that are clamped to the
// matrix, so no load leaves the operand (gemm_mfma_dl_supported keeps the leading dimensions small enough).
// The type only exists in device code; the host pass sees a stand-in with the same interface.
#if defined(__HIP_DEVICE_COMPILE__)
struct TileSource {
  __amdgpu_buffer_rsrc_t rs;
  __device__ __forceinline__ explicit TileSource(const bf16_t *base)
      : rs(__builtin_amdgcn_make_buffer_rsrc((void *)base, 0, 0x7ffffff0, 0x00020000)) {}
  // 16 bytes per lane from base + lane_bytes + uniform_bytes to lds_wave_uniform + 16 * lane
  __device__ __forceinline__ void load16(unsigned lane_bytes, unsigned uniform_bytes, unsigned char *lds_wave_uniform) const {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (__attribute__((address_space(3))) void *)lds_wave_uniform, 16, lane_bytes,
                                             uniform_bytes, 0, 0);
  }
};
#else
struct TileSource {
  __device__ explicit TileSource(const bf16_t *) {}
  __device__ void load16(unsigned, unsigned, unsigned char *) const {}
};
#endif

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order
template <int N, int I = 0, typename F>
__device__ __forceinline__ void unrolled(F &&f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    unrolled<N, I + 1>(f);
  }
}

// Workgroup id -> output tile.  Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2, so XCD x runs
// the ids x, x + 8, ...  Every XCD gets one rectangular block of the tile grid - the grid is cut gx times along M and
// 8 / gx times along N - because what an XCD fetches from memory is the A rows of its block plus the W rows of its
// block: a contiguous run of tiles (a block one tile-column wide and all of M high) makes every XCD fetch all of A
// (Flux-scale MLP-down: 623 MB fetched per launch for 157 MB of operands).  Inside the block the N index runs
// fastest (workgroups in flight together share A tiles; measured equal or better than M fastest on every GEMM of the
// five workloads, up to 12 % on the QKV projections).  Returns false for the surplus ids of the padded grid.
__host__ __device__ __forceinline__ bool tile_of_id(int id, int tiles_m, int tiles_n, int gx, int &tm, int &tn) {
  const int gy = 8 / gx;
  const int bm = (tiles_m + gx - 1) / gx, bn = (tiles_n + gy - 1) / gy;
  const int x = id & 7, j = id >> 3;
  if (j >= bm * bn) return false;
  const int lm = j / bn, ln = j - lm * bn;
  tm = (x % gx) * bm + lm;
  tn = (x / gx) * bn + ln;
  return tm < tiles_m && tn < tiles_n;
}
__device__ __forceinline__ bool tile_of_block(int tiles_m, int tiles_n, int gx, int &tm, int &tn) {
  return tile_of_id(blockIdx.x, tiles_m, tiles_n, gx, tm, tn);
}

// Residual and gate operands of a mode-1 epilogue, fetched by the thread that will use them before the K loop starts, so
// that their memory latency runs under the loop instead of after it (the residual rows were written by an earlier
// kernel and are in no cache).  Only for tiles small enough that a thread owns at most IT 8-column groups.  A tile is
// read and written by its own workgroup only, so reading R early is safe when the GEMM updates it in place.
template <int BM, int BN, int NT>
struct EpiOperands {
  static constexpr int IT = BM * BN / 8 / NT;
  float4 r[IT][2], g[IT][2];
  bool on;
  __device__ __forceinline__ void fetch(int m0, int n0, int M, int N, const Epilogue<bf16_t> &epi, bool vec_ok) {
    on = vec_ok && epi.mode == 1;
    if (!on) return;
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int grp = threadIdx.x + it * NT;
      const int row = m0 + grp / (BN / 8), col = n0 + (grp % (BN / 8)) * 8;
      if (row >= M || col + 8 > N) continue;
      const float *rp = epi.R + (size_t)row * epi.ldr + col;
      r[it][0] = *reinterpret_cast<const float4 *>(rp); r[it][1] = *reinterpret_cast<const float4 *>(rp + 4);
      if (epi.gate) {
        const float *gp = epi.gate_of(row) + col;
        g[it][0] = *reinterpret_cast<const float4 *>(gp); g[it][1] = *reinterpret_cast<const float4 *>(gp + 4);
      }
    }
  }
};

// Epilogue over a finished fp32 tile held row-major in LDS (row stride TLD floats).  PRE: residual / gate operands
// come from `ops` (fetched earlier) when ops->on.
template <int BM, int BN, int TLD, int NT = 256, bool PRE = false>
__device__ __forceinline__ void tile_epilogue(const float *tile, int m0, int n0, int M, int N, const Epilogue<bf16_t> &epi,
                                              bool vec_ok, const EpiOperands<BM, BN, NT> *ops = nullptr) {
  constexpr int GROUPS = BM * BN / 8;
  constexpr int IT = (GROUPS + NT - 1) / NT, UNR = PRE ? IT : 1;
#pragma unroll UNR
  for (int it = 0; it < IT; ++it) {
    const int g = threadIdx.x + it * NT;
    if (GROUPS % NT != 0 && g >= GROUPS) break;
    const int r = g / (BN / 8), c0 = (g % (BN / 8)) * 8;
    const int row = m0 + r, col = n0 + c0;
    if (row >= M || col >= N) continue;
    const float *src = tile + r * TLD + c0;
    float4 lo = *reinterpret_cast<const float4 *>(src), hi4 = *reinterpret_cast<const float4 *>(src + 4);
    float v[8] = {lo.x, lo.y, lo.z, lo.w, hi4.x, hi4.y, hi4.z, hi4.w};
    if (!vec_ok || col + 8 > N) {
      for (int e = 0; e < 8 && col + e < N; ++e) epi.apply(row, col + e, v[e]);
      continue;
    }
    if (epi.bias) {
      bf16x8 b = *reinterpret_cast<const bf16x8 *>(epi.bias + col);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] += (float)b[e];
    }
    if (epi.mode == 0 && epi.kv.kbuf) {
      // QKV projection routed into the K / V^T buffers (an 8-column group never straddles q|k|v or two heads)
      const KvRoute &kv = epi.kv;
      const int part = col / kv.d, cc = col - part * kv.d;
      const int hh = cc / kv.dh, ch = cc - hh * kv.dh;
      const int img = kv.seg > 0 ? row / kv.seg : 0;
      const int lrow = row - img * kv.seg;           // row inside its image
      if (kv.rope && part < 2) {
        const float2 *tab = kv.rope + (size_t)lrow * (kv.dh >> 1) + (ch >> 1);
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          float2 cs = tab[e >> 1];
          float a0 = v[e], b0 = v[e + 1];
          v[e] = a0 * cs.x - b0 * cs.y;
          v[e + 1] = a0 * cs.y + b0 * cs.x;
        }
      }
      if (part == 0 && kv.q_scale != 0.f) {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] *= kv.q_scale;
      }
      bf16x8 o;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = (bf16_t)v[e];
      if (part == 0) {
        *reinterpret_cast<bf16x8 *>(reinterpret_cast<bf16_t *>(epi.C) + (size_t)row * epi.ldc + col) = o;
      } else if (part == 1) {
        const int brow = lrow < kv.split ? kv.row0a + lrow : kv.row0b + (lrow - kv.split);
        *reinterpret_cast<bf16x8 *>(reinterpret_cast<bf16_t *>(kv.kbuf) + (size_t)img * kv.img_stride +
                                    ((size_t)hh * kv.Lp + brow) * kv.dh + ch) = o;
      }
      // part 2 (v) is written by the transposed pass below
    } else if (epi.mode == 0) {
      if (col + 8 > epi.gelu_from) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (col + e >= epi.gelu_from) v[e] = gelu_f(v[e], epi.gelu_tanh);
      }
      bf16x8 o;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = (bf16_t)v[e];
      *reinterpret_cast<bf16x8 *>(reinterpret_cast<bf16_t *>(epi.C) + (size_t)row * epi.ldc + col) = o;
    } else {
      float4 r0, r1, g0, g1;
      bool have = false;
      if constexpr (PRE) {
        if (ops->on) { r0 = ops->r[it][0]; r1 = ops->r[it][1]; g0 = ops->g[it][0]; g1 = ops->g[it][1]; have = true; }
      }
      if (!have) {
        const float *rp = epi.R + (size_t)row * epi.ldr + col;
        r0 = *reinterpret_cast<const float4 *>(rp); r1 = *reinterpret_cast<const float4 *>(rp + 4);
        if (epi.gate) {
          const float *gp = epi.gate_of(row) + col;
          g0 = *reinterpret_cast<const float4 *>(gp); g1 = *reinterpret_cast<const float4 *>(gp + 4);
        }
      }
      float x[8] = {r0.x, r0.y, r0.z, r0.w, r1.x, r1.y, r1.z, r1.w};
      if (epi.gate) {
        float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] += gg[e] * v[e];
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] += v[e];
      }
      float *xp = reinterpret_cast<float *>(epi.C) + (size_t)row * epi.ldc + col;
      *reinterpret_cast<float4 *>(xp) = make_float4(x[0], x[1], x[2], x[3]);
      *reinterpret_cast<float4 *>(xp + 4) = make_float4(x[4], x[5], x[6], x[7]);
      if (epi.C2) {
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = (bf16_t)x[e];
        *reinterpret_cast<bf16x8 *>(epi.C2 + (size_t)row * epi.ldc2 + col) = o;
      }
    }
  }
  // v columns of a routed QKV projection: V^T[h][c][buffer row].  The tile is walked column-wise, eight consecutive
  // rows per thread and consecutive threads along the rows, so that the stores run along V^T's contiguous axis.
  if (epi.mode == 0 && epi.kv.kbuf && n0 + BN > 2 * epi.kv.d) {
    const KvRoute &kv = epi.kv;
    constexpr int RG = BM / 8;
    for (int u = threadIdx.x; u < RG * BN; u += NT) {
      const int rg = u % RG, cl = u / RG;
      const int col = n0 + cl, row = m0 + rg * 8;
      if (col >= N || col < 2 * kv.d || row >= M) continue;
      const int cc = col - 2 * kv.d;
      const float b = epi.bias ? (float)epi.bias[col] : 0.f;
      bf16x8 o;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = (bf16_t)(tile[(rg * 8 + e) * TLD + cl] + b);
      bf16_t *vt = reinterpret_cast<bf16_t *>(kv.vtbuf) + (size_t)cc * kv.Lp;   // cc = h*dh + c; image 0
      const int img = kv.seg > 0 ? row / kv.seg : 0;
      const int lrow = row - img * kv.seg;
      const int brow = lrow < kv.split ? kv.row0a + lrow : kv.row0b + (lrow - kv.split);
      const bool whole = row + 8 <= M && (kv.seg <= 0 || lrow + 8 <= kv.seg) && (lrow >= kv.split || lrow + 8 <= kv.split);
      if (whole && (brow & 7) == 0) {
        *reinterpret_cast<bf16x8 *>(vt + (size_t)img * kv.img_stride + brow) = o;
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int r2 = row + e;
          if (r2 >= M) break;
          const int i2 = kv.seg > 0 ? r2 / kv.seg : 0;
          const int l2 = r2 - i2 * kv.seg;
          vt[(size_t)i2 * kv.img_stride + (l2 < kv.split ? kv.row0a + l2 : kv.row0b + (l2 - kv.split))] = o[e];
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------------------------
// WGM x WGN wavefronts on one shared tile
// ------------------------------------------------------------------------------------------------------------------
template <int BM, int BN, int NSTAGE, int WGM = 2, int WGN = 2, int KB = 64, bool SPREAD_LOADS = false>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_tile_kernel(const bf16_t *__restrict__ A, int64_t lda,
                                                        const bf16_t *__restrict__ W, int64_t ldw, int M, int N, int K,
                                                        Epilogue<bf16_t> epi, int vec_ok, int xcd_gx) {
  constexpr int NW = WGM * WGN;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int MI = WM / 32, NI = WN / 32;
  // KB = K elements per stage: 64 (128-byte tile rows, 8 rows per load instruction, swizzle key (r>>1)&7) or
  // 32 (64-byte rows, 16 rows per instruction, key (r>>2)&3: sixteen consecutive rows then cover all 64 banks)
  constexpr int RBY = KB * 2, RPI = 1024 / RBY, CPR = KB / 8;
  constexpr int LA = BM / RPI / NW, LW = BN / RPI / NW;  // load instructions per wave per stage
  static_assert(BM % (RPI * NW) == 0 && BN % (RPI * NW) == 0, "tile rows must split evenly over the waves' load instructions");
  constexpr int LPS = LA + LW;
  constexpr int STAGE_BYTES = (BM + BN) * RBY;
  auto key = [](int r) { return KB == 64 ? ((r >> 1) & 7) : ((r >> 2) & 3); };
  constexpr int TLD = BN + 4;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WGN, wn = wave % WGN;
  int tm, tn;
  if (!tile_of_block((M + BM - 1) / BM, (N + BN - 1) / BN, xcd_gx, tm, tn)) return;
  const int m0 = tm * BM, n0 = tn * BN;

  // per-lane byte offsets of this wave's load instructions inside the tile's rows (rows past the matrix repeat its last row)
  const TileSource srcA(A + (size_t)m0 * lda), srcW(W + (size_t)n0 * ldw);
  unsigned pa[LA], pw[LW];
#pragma unroll
  for (int i = 0; i < LA; ++i) {
    int r = (i * NW + wave) * RPI + lane / CPR;
    int c = (lane % CPR) ^ key(r);
    pa[i] = (unsigned)(((size_t)min(r, M - 1 - m0) * lda + c * 8) * 2);
  }
#pragma unroll
  for (int i = 0; i < LW; ++i) {
    int r = (i * NW + wave) * RPI + lane / CPR;
    int c = (lane % CPR) ^ key(r);
    pw[i] = (unsigned)(((size_t)min(r, N - 1 - n0) * ldw + c * 8) * 2);
  }
  auto issue = [&](int stage, int kt) {
    unsigned char *sa = smem + stage * STAGE_BYTES;
    unsigned char *sw = sa + BM * RBY;
    const unsigned koff = (unsigned)kt * (KB * 2);
#pragma unroll
    for (int i = 0; i < LA; ++i) srcA.load16(pa[i], koff, sa + (i * NW + wave) * 1024);
#pragma unroll
    for (int i = 0; i < LW; ++i) srcW.load16(pw[i], koff, sw + (i * NW + wave) * 1024);
  };
  // load instruction `idx` (A instructions first, then W) of this wave for K tile kt
  auto issue_one = [&](auto idx_c, int stage, int kt) __attribute__((always_inline)) {
    constexpr int idx = decltype(idx_c)::value;
    unsigned char *sa = smem + stage * STAGE_BYTES;
    const unsigned koff = (unsigned)kt * (KB * 2);
    if constexpr (idx < LA) srcA.load16(pa[idx], koff, sa + (idx * NW + wave) * 1024);
    else srcW.load16(pw[idx - LA], koff, sa + BM * RBY + ((idx - LA) * NW + wave) * 1024);
  };

  // small tiles: the epilogue's residual / gate operands are requested first, ahead of every tile load
  constexpr bool EPRE = BM * BN / 8 / (64 * NW) <= 2;
  EpiOperands<BM, BN, 64 * NW> eops;
  if constexpr (EPRE) eops.fetch(m0, n0, M, N, epi, vec_ok != 0);

  f32x16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = K / KB;
#pragma unroll
  for (int s = 0; s < NSTAGE - 1; ++s)
    if (s < nk) issue(s, s);

  const int l32 = lane & 31, hi = lane >> 5;
  int arow[MI], akey[MI], wrow[NI], wkey[NI];
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    int r = wm * WM + i * 32 + l32;
    arow[i] = r * RBY;
    akey[i] = key(r);
  }
#pragma unroll
  for (int j = 0; j < NI; ++j) {
    int r = wn * WN + j * 32 + l32;
    wrow[j] = BM * RBY + r * RBY;
    wkey[j] = key(r);
  }

  // SPREAD: the loads of the tile that is prefetched during K tile kt are not issued in one burst after the barrier but
  // one at a time between the MFMA groups of the tile (the burst fills the memory pipeline's queue and every wave
  // then stalls at its own load instructions before it can start on its MFMAs).  Every iteration issues the same LPS
  // loads - past the last K tile it repeats the last tile into the stage that has just been freed - so the loop body has
  // no branch around a load and the wait in front of tile kt is the same for every kt.
  constexpr int KS = KB / 16;
  constexpr bool SPREAD = SPREAD_LOADS && MI * NI * KS >= 2 * LPS;
  const int prologue_tiles = min(NSTAGE - 1, nk);
  for (int kt = 0; kt < nk; ++kt) {
    // tiles still in flight behind tile kt: min(NSTAGE-2, nk-1-kt); wait until only their loads are outstanding
    const int behind = SPREAD ? prologue_tiles - 1 : min(NSTAGE - 2, nk - 1 - kt);
    wait_tiles_behind<LPS, NSTAGE - 2>(behind);
    // plain s_barrier: __syncthreads() would also drain every global load in flight (vmcnt(0)), i.e. the prefetches
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    const int ld_stage = (kt + NSTAGE - 1) % NSTAGE, ld_kt = min(kt + NSTAGE - 1, nk - 1);
    if constexpr (!SPREAD) {
      if (kt + NSTAGE - 1 < nk) issue(ld_stage, kt + NSTAGE - 1);
    }
    const unsigned char *st = smem + (kt % NSTAGE) * STAGE_BYTES;
    // Fragments are read from LDS PRE k-steps ahead of the MFMAs that use them: with one accumulator per wave
    // (64x64 tile) a k-step is a single MFMA, far shorter than an LDS read, so the whole tile is preloaded.
    constexpr int PRE = (MI * NI <= 2) ? KS : 2;
    bf16x8 af[PRE][MI], wf[PRE][NI];
    auto lread = [&](int buf, int ks) {
      const int c = ks * 2 + hi;
#pragma unroll
      for (int i = 0; i < MI; ++i) af[buf][i] = *reinterpret_cast<const bf16x8 *>(st + arow[i] + ((c ^ akey[i]) << 4));
#pragma unroll
      for (int j = 0; j < NI; ++j) wf[buf][j] = *reinterpret_cast<const bf16x8 *>(st + wrow[j] + ((c ^ wkey[j]) << 4));
    };
#pragma unroll
    for (int ks = 0; ks < PRE - 1; ++ks) lread(ks, ks);
    unrolled<KS>([&](auto ks_c) __attribute__((always_inline)) {
      constexpr int ks = decltype(ks_c)::value;
      if (ks + PRE - 1 < KS) lread((ks + PRE - 1) % PRE, ks + PRE - 1);
      // keep the LDS reads of the next k-step ahead of this k-step's MFMAs (the scheduler would otherwise sink them
      // to reuse the fragment registers, exposing the LDS latency at every k-step)
      __builtin_amdgcn_sched_barrier(0);
      unrolled<MI * NI>([&](auto m_c) __attribute__((always_inline)) {
        constexpr int m = decltype(m_c)::value, i = m / NI, j = m % NI;
        if constexpr (SPREAD) {
          // MFMA number g of the tile's G = MI * NI * KS; load l goes in front of MFMA (2 l + 1) G / (2 LPS)
          constexpr int g = ks * MI * NI + m, G = MI * NI * KS;
          constexpr int l = g * LPS / G;
          if constexpr (l < LPS && g == ((2 * l + 1) * G) / (2 * LPS)) {
            issue_one(std::integral_constant<int, l>{}, ld_stage, ld_kt);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks % PRE][i], wf[ks % PRE][j], acc[i][j], 0, 0, 0);
      });
    });
  }

  // accumulators -> row-major fp32 tile in LDS (lane -> column l32, register r -> row 8*(r/4) + 4*hi + r%4), in
  // passes of RB rows when the whole tile does not fit in the stage memory
  constexpr int RING = NSTAGE * STAGE_BYTES;
  constexpr int RB = (BM * TLD * 4 <= RING) ? BM : ((BM / 2) * TLD * 4 <= RING ? BM / 2 : BM / 4);
  static_assert(RB * TLD * 4 <= RING || RB == BM, "epilogue pass does not fit");
  static_assert(RB % WM == 0 || WM % RB == 0, "pass rows and wave rows must nest");
  float *tile = reinterpret_cast<float *>(smem);
#pragma unroll
  for (int pass = 0; pass < BM / RB; ++pass) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const int rbase = wm * WM + i * 32;          // first tile row of this 32-row block
      if (rbase / RB != pass) continue;
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          tile[(rbase - pass * RB + 8 * (r >> 2) + 4 * hi + (r & 3)) * TLD + wn * WN + j * 32 + l32] = acc[i][j][r];
    }
    __syncthreads();
    if constexpr (EPRE && RB == BM) tile_epilogue<BM, BN, TLD, 64 * NW, true>(tile, m0, n0, M, N, epi, vec_ok != 0, &eops);
    else tile_epilogue<RB, BN, TLD, 64 * NW>(tile, m0 + pass * RB, n0, M, N, epi, vec_ok != 0);
  }
}

// ------------------------------------------------------------------------------------------------------------------
// four wavefronts split K; each owns a private two-stage ring for its own BM x BN x 64 tiles
// ------------------------------------------------------------------------------------------------------------------
template <int BM, int BN>
__global__ __launch_bounds__(256) void gemm_wavek_kernel(const bf16_t *__restrict__ A, int64_t lda,
                                                         const bf16_t *__restrict__ W, int64_t ldw, int M, int N, int K,
                                                         Epilogue<bf16_t> epi, int vec_ok, int xcd_gx) {
  constexpr int MI = BM / 32, NI = BN / 32;
  constexpr int LA = BM / 8, LW = BN / 8;   // load instructions per wave per stage (a wave loads whole tiles)
  constexpr int LPS = LA + LW;
  constexpr int STAGE_BYTES = (BM + BN) * ROW_BYTES;
  constexpr int WAVE_BYTES = 2 * STAGE_BYTES;
  constexpr int TLD = BN + 4;
  static_assert(LPS <= 31, "two stages of loads must fit the vmcnt counter");
  static_assert(WAVE_BYTES >= BM * TLD * 4, "a wave's partial tile must fit in its own ring");
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  int tm, tn;
  if (!tile_of_block((M + BM - 1) / BM, (N + BN - 1) / BN, xcd_gx, tm, tn)) return;
  const int m0 = tm * BM, n0 = tn * BN;
  unsigned char *ring = smem + wave * WAVE_BYTES;

  // K tiles of this wave: wave, wave + 4, ...
  const int nk = K / BK;
  const int my_nk = (nk - wave + 3) / 4;

  const int lr = lane >> 3, lc = lane & 7;
  const TileSource srcA(A + (size_t)m0 * lda), srcW(W + (size_t)n0 * ldw);
  unsigned pa[LA], pw[LW];   // per-lane byte offsets inside the tile's rows; instruction i covers tile rows 8i .. 8i+7
#pragma unroll
  for (int i = 0; i < LA; ++i) {
    int r = i * 8 + lr;
    int c = lc ^ ((r >> 1) & 7);
    pa[i] = (unsigned)(((size_t)min(r, M - 1 - m0) * lda + c * 8) * 2);
  }
#pragma unroll
  for (int i = 0; i < LW; ++i) {
    int r = i * 8 + lr;
    int c = lc ^ ((r >> 1) & 7);
    pw[i] = (unsigned)(((size_t)min(r, N - 1 - n0) * ldw + c * 8) * 2);
  }
  auto issue = [&](int stage, int t) {   // t-th tile of this wave
    unsigned char *sa = ring + stage * STAGE_BYTES;
    unsigned char *sw = sa + BM * ROW_BYTES;
    const unsigned koff = (unsigned)(wave + 4 * t) * (BK * 2);
#pragma unroll
    for (int i = 0; i < LA; ++i) srcA.load16(pa[i], koff, sa + i * 1024);
#pragma unroll
    for (int i = 0; i < LW; ++i) srcW.load16(pw[i], koff, sw + i * 1024);
  };

  f32x16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  constexpr bool EPRE = BM * BN / 8 / 256 <= 2 && BM * BN / 8 >= 256;
  EpiOperands<BM, BN, 256> eops;
  if constexpr (EPRE) eops.fetch(m0, n0, M, N, epi, vec_ok != 0);

  if (my_nk > 0) issue(0, 0);
  if (my_nk > 1) issue(1, 1);

  const int l32 = lane & 31, hi = lane >> 5;
  for (int t = 0; t < my_nk; ++t) {
    if (t + 1 < my_nk) wait_vmcnt<LPS>(); else wait_vmcnt<0>();
    asm volatile("" ::: "memory");
    const unsigned char *st = ring + (t & 1) * STAGE_BYTES;
    bf16x8 af[2][MI], wf[2][NI];
    auto lread = [&](int buf, int ks) {
      const int c = ks * 2 + hi;
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        int r = i * 32 + l32;
        af[buf][i] = *reinterpret_cast<const bf16x8 *>(st + r * ROW_BYTES + ((c ^ ((r >> 1) & 7)) << 4));
      }
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        int r = j * 32 + l32;
        wf[buf][j] = *reinterpret_cast<const bf16x8 *>(st + (BM + r) * ROW_BYTES + ((c ^ ((r >> 1) & 7)) << 4));
      }
    };
    lread(0, 0);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      if (ks + 1 < BK / 16) lread((ks + 1) & 1, ks + 1);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][i], wf[ks & 1][j], acc[i][j], 0, 0, 0);
    }
    // this wave's LDS reads of the stage are complete (the MFMAs above consumed them): refill it
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (t + 2 < my_nk) issue(t & 1, t + 2);
  }

  // partial tiles -> LDS (each wave into its own ring), then sum of the four and epilogue
  float *part = reinterpret_cast<float *>(ring);
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        part[(i * 32 + 8 * (r >> 2) + 4 * hi + (r & 3)) * TLD + j * 32 + l32] = acc[i][j][r];
  __syncthreads();
  float *p0 = reinterpret_cast<float *>(smem);
  constexpr int WSTRIDE = WAVE_BYTES / 4;
  for (int e = tid; e < BM * BN / 4; e += 256) {
    int r = e / (BN / 4), c = (e % (BN / 4)) * 4;
    float4 s0 = *reinterpret_cast<const float4 *>(p0 + r * TLD + c);
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      float4 s1 = *reinterpret_cast<const float4 *>(p0 + w * WSTRIDE + r * TLD + c);
      s0.x += s1.x; s0.y += s1.y; s0.z += s1.z; s0.w += s1.w;
    }
    *reinterpret_cast<float4 *>(p0 + r * TLD + c) = s0;
  }
  __syncthreads();
  if constexpr (EPRE) tile_epilogue<BM, BN, TLD, 256, true>(p0, m0, n0, M, N, epi, vec_ok != 0, &eops);
  else tile_epilogue<BM, BN, TLD>(p0, m0, n0, M, N, epi, vec_ok != 0);
}

// Cut of the tile grid over the 8 XCDs (see tile_of_block): the gx in {1, 2, 4, 8} for which an XCD's block needs the
// fewest operand rows; a cut that pads the grid by more than an eighth is priced four times.  *grid receives the
// workgroup count.
int xcd_cut(const GemmArgs &a, int BM, int BN, unsigned *grid) {
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  int best = 1;
  double best_cost = 1e300;
  const int64_t T = (int64_t)tiles_m * tiles_n;
  for (int gx = 1; gx <= 8; gx *= 2) {
    const int gy = 8 / gx;
    const int bm = (tiles_m + gx - 1) / gx, bn = (tiles_n + gy - 1) / gy;
    const int64_t padded = 8LL * bm * bn;
    double cost = (double)bm * BM + (double)bn * BN;          // operand rows per XCD (both operands have K columns)
    if (padded * 8 > T * 9) cost *= 4.0;                       // too many idle workgroup slots
    if (cost < best_cost) { best_cost = cost; best = gx; }
  }
  const int gy = 8 / best;
  const int bm = (tiles_m + best - 1) / best, bn = (tiles_n + gy - 1) / gy;
  *grid = (unsigned)(8 * bm * bn);
  return best;
}

}  // namespace

// Host view of the workgroup -> tile map of a launch with BM x BN tiles (what workgroup `id` of the kernel computes):
// the grid size in *grid, and whether `id` has a tile (then in *tm, *tn).  For the unit test of the map.
bool gemm_tile_map(int M, int N, int BM, int BN, unsigned id, unsigned *grid, int *tm, int *tn) {
  GemmArgs a{};
  a.M = M; a.N = N;
  const int gx = xcd_cut(a, BM, BN, grid);
  if (id >= *grid) return false;
  return tile_of_id((int)id, (M + BM - 1) / BM, (N + BN - 1) / BN, gx, *tm, *tn);
}

namespace {

bool vec_epilogue_ok(const GemmArgs &a) {
  auto al = [](const void *p, uintptr_t n) { return ((uintptr_t)p % n) == 0; };
  bool ok = (!a.bias || al(a.bias, 16));
  if (a.epilogue == 0) return ok && al(a.C, 16) && a.ldc % 8 == 0;
  ok = ok && al(a.C, 16) && a.ldc % 4 == 0 && al(a.R, 16) && a.ldr % 4 == 0 && (!a.gate || (al(a.gate, 16) && a.gate_stride % 4 == 0));
  if (a.C2) ok = ok && al(a.C2, 16) && a.ldc2 % 8 == 0;
  return ok;
}

template <int BM, int BN, int NSTAGE, int WGM = 2, int WGN = 2, int KB = 64, bool SPREAD = false>
hipError_t launch_tile(const GemmArgs &a, hipStream_t s) {
  // the stage ring, or the fp32 tile (row stride BN + 4) that replaces it for the epilogue, whichever is larger
  constexpr int ring = NSTAGE * (BM + BN) * KB * 2, tile = BM * (BN + 4) * 4;
  constexpr int smem = (tile > ring && tile <= 96 * 1024) ? tile : ring;   // larger tiles finish in row passes
  if (hipError_t e = allow_dynamic_lds<&gemm_tile_kernel<BM, BN, NSTAGE, WGM, WGN, KB, SPREAD>, smem>(); e != hipSuccess) return e;
  unsigned grid = 0;
  const int gx = xcd_cut(a, BM, BN, &grid);
  dim3 g(grid);
  gemm_tile_kernel<BM, BN, NSTAGE, WGM, WGN, KB, SPREAD><<<g, 64 * WGM * WGN, smem, s>>>((const bf16_t *)a.A, a.lda, (const bf16_t *)a.W, a.ldw, a.M, a.N,
                                                       a.K, make_epilogue<bf16_t>(a), vec_epilogue_ok(a) ? 1 : 0, gx);
  return hipGetLastError();
}

template <int BM, int BN>
hipError_t launch_wavek(const GemmArgs &a, hipStream_t s) {
  constexpr int smem = 4 * 2 * (BM + BN) * ROW_BYTES;
  if (hipError_t e = allow_dynamic_lds<&gemm_wavek_kernel<BM, BN>, smem>(); e != hipSuccess) return e;
  unsigned grid = 0;
  const int gx = xcd_cut(a, BM, BN, &grid);
  dim3 g(grid);
  gemm_wavek_kernel<BM, BN><<<g, 256, smem, s>>>((const bf16_t *)a.A, a.lda, (const bf16_t *)a.W, a.ldw, a.M, a.N, a.K,
                                                make_epilogue<bf16_t>(a), vec_epilogue_ok(a) ? 1 : 0, gx);
  return hipGetLastError();
}

}  // namespace

bool gemm_kv_route_supported(const GemmArgs &a) {
  return a.dt == DT_BF16 && a.path != PATH_SIMT && a.epilogue == 0 && a.K % BK == 0 && a.K >= BK && a.N % 8 == 0 &&
         vec_epilogue_ok(a) && a.kvr.dh % 8 == 0 && a.kvr.d % 8 == 0 && a.N == 3 * a.kvr.d;
}

// (the tile loads address a tile's rows with 32-bit byte offsets inside a 2 GB window: 256 rows of either operand must fit)
bool gemm_mfma_dl_supported(const GemmArgs &a) {
  const int64_t ld = a.lda > a.ldw ? a.lda : a.ldw;
  return a.K % BK == 0 && a.K >= BK && a.M >= 1 && a.N >= 1 && (256 * ld + a.K) * 2 < 0x7ffffff0LL;
}

// Tile heuristic, from A/B runs inside the stage on MI355X (weights come from HBM there, not from a warm L2, which
// favours deeper rings than an isolated GEMM loop suggests):
//  * the 8-wave 256x256 / 256x128 tiles need the fewest L1 bytes per flop and win once they fill the chip;
//    256x128 runs best with 32-wide K stages and three of them; long-K GEMMs with few tiles (Flux-scale MLP-down:
//    192 tiles, K = 15360) prefer it too, with 64-wide stages;
//  * 128x128 (two workgroups per CU) from about 1.5 workgroups per CU, then 128x64;
//  * skinny GEMMs (n = 512 patch rows): 64x64 tiles, four stages while every workgroup is resident at once (two per CU:
//    up to 512 tiles), two stages (five per CU) beyond - the three-stage ring that used to sit between them lost its
//    edge once the stage's weights stayed in the memory-side cache (SD3-scale MLP-up, 768 tiles: 21.9 -> 20.9 us) -
//    and the K-splitting kernel when K is long and tiles are few;
//  * 192-wide tiles (three 32-column blocks per wave) when they cut the output into a whole number of 256-workgroup
//    rounds, which power-of-two tiles cannot do for widths that are multiples of 3 * 1024 (Flux-scale stage, patch of
//    2048 rows: QKV 171 -> 144 us with 768 tiles of 128x192, MLP-up 178 -> 172 us with 512 tiles of 256x192, MLP-down
//    241 -> 214 us with 256 tiles of 128x192 and three stages); not for K = 1152, where the two-stage ring is exposed.
//  * the three-stage 128x192 tile (long K, few tiles) issues its prefetch loads one at a time between the MFMAs of the
//    tile instead of in a burst after the barrier (isolated GEMM, interleaved A/B rounds: 2048x3072x15360 204 -> 183 us,
//    4096x1152x4608 65 -> 55 us; inside the Flux-scale stage 225 -> 193 us).  The other tiles keep the burst: the
//    two-stage 128x192 tile gains alone (2048x9216x3072 129 -> 122 us) but not inside the stage (150 -> 154 us), the
//    8-wave tiles and the 64x64 tiles lose (256x192: 152 -> 171 us, 256x256 at 8192^3: 995 -> 1063 us, 64x64: 15.2 ->
//    17.7 us).
enum { V_256x256 = 0, V_256x128_K32S3, V_256x128_S3, V_128x128, V_128x64, V_WAVEK, V_64x64_S4, V_64x64_S3, V_64x64_S2,
       V_128x192_S2, V_256x192_S2, V_128x192_S3, V_COUNT };

static int pick_variant(const GemmArgs &a) {
  auto tiles = [&](int bm, int bn) { return (int64_t)((a.M + bm - 1) / bm) * ((a.N + bn - 1) / bn); };
  if (a.N % 192 == 0 && a.M % 128 == 0) {
    const int64_t t192 = tiles(128, 192);
    if (a.K >= 4096 && t192 >= 128 && t192 <= 256) return V_128x192_S3;
    // shorter K: only with enough rounds that the two-stage ring's exposed start is amortised (PixArt MLP-up on a
    // 4096-row patch, 768 tiles: 104 -> 89 us)
    if (a.K >= 1024 && a.K < 2048 && t192 % 256 == 0 && t192 >= 512 && t192 <= 1024) return V_128x192_S2;
    if (a.K >= 2048 && t192 % 256 == 0 && t192 <= 1024) {
      const int64_t t2 = a.M % 256 == 0 ? tiles(256, 192) : 0;
      return (t2 >= 512 && t2 % 256 == 0) ? V_256x192_S2 : V_128x192_S2;
    }
  }
  if (tiles(256, 256) >= 1024) return V_256x256;
  if (tiles(256, 128) >= 512) return V_256x128_K32S3;
  if (a.K >= 8192 && tiles(256, 128) >= 128) return V_256x128_S3;
  if (tiles(128, 128) >= 384) return V_128x128;
  if (tiles(128, 64) >= 512) return V_128x64;
  const int64_t t64 = tiles(64, 64);
  if (t64 < g_wavek_max_tiles && a.K >= g_wavek_min_k) return V_WAVEK;
  // one tile per CU at most (the d x d projections of a 512-row patch): the wave-split-K kernel from K = 1024 on
  // (inside the stage: PixArt-scale cross projections 9.3 -> 8.6 us, SD3-scale out-projection 11.8 -> 10.8 us; with
  // more tiles than CUs it loses: PixArt-scale QKV 13.2 -> 17.9 us)
  if (t64 <= 256 && a.K >= 1024) return V_WAVEK;
  if (t64 <= 512) return V_64x64_S4;
  return V_64x64_S2;
}

static hipError_t launch_variant(int v, const GemmArgs &a, hipStream_t s) {
  switch (v) {
    case V_256x256: return launch_tile<256, 256, 2, 4, 2>(a, s);
    case V_256x128_K32S3: return launch_tile<256, 128, 3, 4, 2, 32>(a, s);
    case V_256x128_S3: return launch_tile<256, 128, 3, 4, 2>(a, s);
    case V_128x128: return launch_tile<128, 128, 2>(a, s);
    case V_128x64: return launch_tile<128, 64, 2>(a, s);
    case V_WAVEK: return launch_wavek<64, 64>(a, s);
    case V_64x64_S4: return launch_tile<64, 64, 4>(a, s);
    case V_64x64_S3: return launch_tile<64, 64, 3>(a, s);
    case V_128x192_S2: return launch_tile<128, 192, 2>(a, s);
    case V_256x192_S2: return launch_tile<256, 192, 2, 4, 2>(a, s);
    case V_128x192_S3: return launch_tile<128, 192, 3, 2, 2, 64, true>(a, s);
    default: return launch_tile<64, 64, 2>(a, s);
  }
}

int gemm_mfma_dl_tile_count() { return V_COUNT; }

hipError_t launch_gemm_mfma_dl(const GemmArgs &a, hipStream_t s) {
#ifdef PF_TUNING
  // tile configurations outside the heuristic's set, for sweeps
  switch (g_gemm_tile_override) {
    case 1: return launch_tile<256, 128, 3>(a, s);
    case 2: return launch_tile<128, 128, 3>(a, s);
    case 3: return launch_tile<128, 128, 2>(a, s);
    case 4: return launch_tile<128, 64, 4>(a, s);
    case 5: return launch_tile<64, 64, 4>(a, s);
    case 6: return launch_tile<256, 128, 2>(a, s);
    case 7: return launch_tile<128, 64, 2>(a, s);
    case 8: return launch_tile<64, 64, 2>(a, s);
    case 9: return launch_gemm_mfma(a, s);
    case 10: return launch_wavek<64, 64>(a, s);
    case 14: return launch_tile<256, 128, 3, 4, 2>(a, s);
    case 15: return launch_tile<256, 256, 2, 4, 2>(a, s);
    case 16: return launch_tile<128, 256, 3, 2, 4>(a, s);
    case 17: return launch_tile<256, 128, 2, 4, 2>(a, s);
    case 22: return launch_tile<256, 128, 3, 4, 2, 32>(a, s);
    case 26: return launch_tile<64, 64, 3>(a, s);
    case 27: return launch_tile<128, 64, 3>(a, s);
    case 28: return launch_tile<128, 192, 2>(a, s);
    case 29: return launch_tile<256, 192, 2, 4, 2>(a, s);
    case 30: return launch_tile<128, 192, 3>(a, s);
    case 40: return launch_tile<128, 192, 2, 2, 2, 64, true>(a, s);
    case 41: return launch_tile<256, 192, 2, 4, 2, 64, true>(a, s);
    case 42: return launch_tile<128, 192, 3, 2, 2, 64, true>(a, s);
    case 43: return launch_tile<256, 256, 2, 4, 2, 64, true>(a, s);
    case 44: return launch_tile<256, 128, 3, 4, 2, 64, true>(a, s);
    case 45: return launch_tile<128, 128, 2, 2, 2, 64, true>(a, s);
    case 46: return launch_tile<128, 192, 4, 2, 2, 64, true>(a, s);
    case 47: return launch_tile<128, 128, 3, 2, 2, 64, true>(a, s);
    case 48: return launch_tile<128, 128, 4, 2, 2, 64, true>(a, s);
    case 49: return launch_tile<128, 64, 4, 2, 2, 64, true>(a, s);
    case 50: return launch_tile<64, 64, 4, 2, 2, 64, true>(a, s);
    case 51: return launch_tile<128, 256, 3, 2, 2, 64, true>(a, s);
    case 52: return launch_tile<128, 192, 3, 2, 2, 64, false>(a, s);
    default: break;
  }
#endif
  if (a.tile >= 1 && a.tile <= V_COUNT) return launch_variant(a.tile - 1, a, s);
  return launch_variant(pick_variant(a), a, s);
}

const char *gemm_mfma_dl_variant_name(const GemmArgs &a) {
  static const char *names[V_COUNT] = {"gemm_tile_kernel<256,256,2,4,2,64,false>", "gemm_tile_kernel<256,128,3,4,2,32,false>",
                                       "gemm_tile_kernel<256,128,3,4,2,64,false>", "gemm_tile_kernel<128,128,2,2,2,64,false>",
                                       "gemm_tile_kernel<128,64,2,2,2,64,false>", "gemm_wavek_kernel<64,64>",
                                       "gemm_tile_kernel<64,64,4,2,2,64,false>", "gemm_tile_kernel<64,64,3,2,2,64,false>",
                                       "gemm_tile_kernel<64,64,2,2,2,64,false>", "gemm_tile_kernel<128,192,2,2,2,64,false>",
                                       "gemm_tile_kernel<256,192,2,4,2,64,false>", "gemm_tile_kernel<128,192,3,2,2,64,true>"};
  return names[(a.tile >= 1 && a.tile <= V_COUNT) ? a.tile - 1 : pick_variant(a)];
}

}  // namespace pf
