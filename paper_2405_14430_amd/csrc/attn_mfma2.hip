// Flash-style patch attention for gfx950, head sizes 64 / 72 / 128 (bf16 operands, fp32 accumulation and softmax).
//
// The patch's queries attend over ALL rows of the layer's K/V buffer, fresh and stale alike (PipeFusion Sec. 3.3).
// Per workgroup: 32 queries per wavefront, 4 wavefronts (128 queries, two workgroups per CU) or 8 (256 queries, one
// workgroup per CU whose K/V tiles then serve twice as many queries: half the L2 -> LDS bytes per flop, and the LDS that
// a second workgroup would need goes into a deeper ring), of one head and one split of the key range.  The layout is
// the transposed one (a lane owns one query column):
//   S^T[kv][q] = K[kv][:] . Q[q][:]        A = K tile (LDS), B = Q fragments (registers)
//   O^T[c][q] += V^T[c][kv] . P^T[kv][q]   A = V^T tile (LDS), B = P^T straight from the S^T accumulator registers
// so the online-softmax statistics are in-lane reductions plus one exchange with lane^32 and the O^T rescale is per lane.
//
// K tiles ([64 kv][dh], contiguous in the head-major buffer) and V^T tiles ([dh][64 kv]) come in with
// global_load_lds_dwordx4 into a two- to four-stage LDS ring (one s_barrier per tile, the next one or two tiles in flight
// during tile t).  The LDS side of those loads is lane-linear, so bank conflicts are handled by XOR-swizzling the 16-byte chunks of a
// row (the loading lane fetches the chunk that belongs at its LDS slot); dh = 72 rows are 144 bytes, which is conflict
// free without a swizzle.  Before the PV product the two half-waves exchange half of their packed P registers
// (v_permlane32_swap) so that each lane's eight P values cover eight CONSECUTIVE kv rows; the matching V^T operand is
// then a single 16-byte LDS read.  Workgroup ids are remapped so that all workgroups of one head run on the same XCD and share
// its L2 for that head's K/V.
#include <type_traits>

#include "common.h"
#include "ops.h"

namespace pf {

#ifdef PF_TUNING
// Timeline probe of a tuning build: shader-clock stamps at the phase boundaries of one outer loop iteration (four tile
// steps) of every wave of workgroup 0 of the 8-wave kernel, read back with pf_attn_trace_read.
__device__ unsigned long long g_attn_trace[8][24];
#define PF_STAMP(slot) do { if (tracing) ts[slot] = clock64(); } while (0)
#else
#define PF_STAMP(slot) do { } while (0)
#endif

namespace {

constexpr int TK = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// K / V^T tile loads carry the non-temporal hint (cache-policy bit 1): a call streams every layer's whole K/V through the
// chip once, and with the default policy that stream displaces the stage's weights from the L2s and the memory-side
// cache; the GEMMs of a stage whose weights fit there run 8 - 10 % faster behind an attention launch that streams
// (SD3-scale call 0.357 -> 0.336 ms, PixArt-scale 0.452 -> 0.440 ms; the kernel itself and the Flux-scale call, whose
// weights do not fit anyway, measure the same).  The workgroups of a head still share its tiles through their XCD's L2.
constexpr int kTileLoadPolicy = 2;
// Tile loads are raw-buffer loads into LDS: a wave-uniform resource over one head's K (or V^T), a wave-uniform byte
// offset (tile, instruction) and one 32-bit per-lane byte offset, so a load costs no 64-bit per-lane address arithmetic
// on the vector unit (which a matrix phase would take from the partner wave's softmax).  The resource spans 2 GB from
// the head's first element; a head's K and V^T are far smaller (the host checks rows_padded < 2^23) and every offset
// stays inside the head.  The type only exists in device code; the host pass sees a stand-in.
#if defined(__HIP_DEVICE_COMPILE__)
struct HeadSource {
  __amdgpu_buffer_rsrc_t rs;
  __device__ __forceinline__ explicit HeadSource(const void *base)
      : rs(__builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, 0x7ffffff0, 0x00020000)) {}
  // 16 bytes per lane from base + lane_bytes + uniform_bytes to lds_wave_uniform + 16 * lane
  __device__ __forceinline__ void load16(unsigned lane_bytes, unsigned uniform_bytes, unsigned char *lds_wave_uniform) const {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (__attribute__((address_space(3))) void *)lds_wave_uniform, 16, lane_bytes,
                                             uniform_bytes, 0, kTileLoadPolicy);
  }
};
#else
struct HeadSource {
  __device__ explicit HeadSource(const void *) {}
  __device__ void load16(unsigned, unsigned, unsigned char *) const {}
};
#endif

// LDS fragment reads whose completion is tracked by hand.  The compiler's own wait insertion is of no use in the tile
// loop: with an LDS-DMA load in flight (there always is one) it treats the LDS counter as unordered and waits for
// lgkmcnt(0) - every outstanding read - in front of an MFMA instead of for that MFMA's fragment.  The read is issued in
// inline assembly, address = (base ^ XOR) + OFF with both constants in the instruction stream (no loop-invariant address
// registers), and lds_wait<N>(frag) waits until at most N LDS operations younger than frag's read are outstanding
// (LDS returns in order; operations of other kinds in between only make the wait longer).  The fragment passes through
// the wait as an in/out operand, so its first use cannot be scheduled in front of it.
template <int XOR, int OFF>
__device__ __forceinline__ bf16x8 lds_read16_async(unsigned base) {
  bf16x8 v;
  static_assert(OFF >= 0, "byte offset");
  if constexpr (XOR == 0 && OFF <= 65535) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(base), "n"(OFF) : "memory");
  } else if constexpr (XOR == 0) {
    unsigned tmp;
    asm volatile("v_add_u32 %1, %3, %2\n\tds_read_b128 %0, %1" : "=&v"(v), "=&v"(tmp) : "v"(base), "n"(OFF) : "memory");
  } else if constexpr (OFF <= 65535) {
    unsigned tmp;
    asm volatile("v_xor_b32 %1, %3, %2\n\tds_read_b128 %0, %1 offset:%4" : "=&v"(v), "=&v"(tmp) : "v"(base), "n"(XOR), "n"(OFF) : "memory");
  } else {
    unsigned tmp;
    asm volatile("v_xor_b32 %1, %3, %2\n\tv_add_u32 %1, %4, %1\n\tds_read_b128 %0, %1"
                 : "=&v"(v), "=&v"(tmp) : "v"(base), "n"(XOR), "n"(OFF) : "memory");
  }
  return v;
}
__device__ __forceinline__ unsigned lds_address(const unsigned char *p) {
  return (unsigned)(uintptr_t)((const __attribute__((address_space(3))) unsigned char *)p);
}
template <int N>
__device__ __forceinline__ void lds_wait(bf16x8 &frag) {
  asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(frag) : "n"(N) : "memory");
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order
template <int N, int I = 0, typename F>
__device__ __forceinline__ void unrolled(F &&f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    unrolled<N, I + 1>(f);
  }
}

// Spread of LH load instructions over a matrix phase of NF MFMAs: load j goes in front of MFMA ((2j + 1) NF) / (2 LH).
// Returns the load that goes in front of MFMA i, or -1.
constexpr int spread_slot(int i, int NF, int LH) {
  for (int j = 0; j < LH; ++j)
    if (((2 * j + 1) * NF) / (2 * LH) == i) return j;
  return -1;
}
static_assert(spread_slot(2, 16, 4) == 0 && spread_slot(14, 16, 4) == 3 && spread_slot(3, 16, 4) == -1, "one load every fourth MFMA");
static_assert(spread_slot(1, 8, 3) == 0 && spread_slot(4, 8, 3) == 1 && spread_slot(6, 8, 3) == 2, "distinct slots");

template <int DH, int NW = 4>
struct Cfg {
  static constexpr int TQ = 32 * NW;                     // queries per workgroup
  static constexpr int KS16 = DH / 16;
  static constexpr bool TAIL8 = (DH % 16) == 8;
  static constexpr int KROW = DH * 2;                    // bytes per K tile row
  static constexpr int KCHUNKS = DH / 8;                 // 16-byte chunks per K row
  static constexpr int K_BYTES = TK * KROW;
  static constexpr int K_INSTR = K_BYTES / 1024;         // 1 KB per load instruction
  static constexpr int CB = (DH + 31) / 32;
  static constexpr int V_ROWS = CB * 32;
  static constexpr int V_BYTES = V_ROWS * 128;
  static constexpr int V_INSTR = DH / 8;                 // 8 rows of 128 B per instruction
  static constexpr int STAGE = K_BYTES + V_BYTES;
  // Waves that issue the tile loads: all four of the 4-wave kernel; in the 8-wave kernel only waves 0..3, which reach the
  // tile's barrier with time to spare (waves 4..7 are the critical path of a tile and issue none).
  static constexpr int NWL = NW == 8 ? 4 : NW;
  static constexpr int LK = (K_INSTR + NWL - 1) / NWL, LV = (V_INSTR + NWL - 1) / NWL;   // instructions per loading wave
  static constexpr int LPS = LK + LV;
  // Head sizes that leave padding rows in the V^T tile (72 -> 96 rows) get the softmax denominator for free: padding
  // row DH holds ones, so row DH of O^T accumulates sum_j P[j][q] in the matrix pipe (with the same rescaling as the
  // numerator) and the per-element additions of the running sum disappear from the VALU stream.
  static constexpr bool ONES_ROW = V_ROWS > DH;
  // swizzle key of K row r (applied to the chunk index)
  static __device__ __forceinline__ int kkey(int r) {
    return DH == 64 ? ((r >> 1) & 7) : (DH == 128 ? (r & 15) : 0);
  }
};

// PRE: the queries arrive already multiplied by log2(e) / sqrt(dh) (the producer folds the factor into its fp32
// epilogue, so q is rounded to bf16 once either way; scaling bf16 queries here would round them a second time and
// costs accuracy on peaked softmaxes).  The score MFMAs then deliver exponents of 2 and the softmax of an element
// needs no multiply-add.
template <int DH, int NS, bool PRE, int NW = 4>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void attn_mfma2_kernel(const bf16_t *__restrict__ q, int64_t ldq,
                                                            const bf16_t *__restrict__ kbuf,
                                                            const bf16_t *__restrict__ vtbuf, int kv_rows, int Lp, int H,
                                                            bf16_t *__restrict__ out, int64_t ldo, int nq, int splits,
                                                            int qtiles, float *__restrict__ ws, int hpi) {
  // H counts heads over all images of the call (image-major, hpi heads per image); q / out rows are image-major too
  using C = Cfg<DH, NW>;
  constexpr int TQ = C::TQ, NT = 64 * NW;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  // LDS ring: the NS K tiles first, then the NS V^T tiles.  Every K fragment then lies within 64 KB of the ring's start
  // and every V^T fragment within 64 KB of the first V^T tile, the reach of an LDS read's offset field, also in the
  // 128 KB ring of the 8-wave dh = 128 kernel.
  constexpr int VRING = NS * C::K_BYTES;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hi = lane >> 5;

  // ---- workgroup id -> (head, query tile, split), heads grouped per XCD (ids are dealt round-robin to the 8 XCDs)
  const int total = gridDim.x;
  int L = blockIdx.x;
  const int per_xcd = total >> 3;
  if (L < per_xcd * 8) L = (L & 7) * per_xcd + (L >> 3);
  const int per_head = qtiles * splits;
  const int h = L / per_head;
  const int rem = L - h * per_head;
  const int qt = rem / splits, sp = rem - qt * splits;
  const int q0 = qt * TQ + wave * 32;

  // ---- zero the V^T padding rows (never written by the tile loads) of every stage
  if constexpr (C::V_ROWS > DH) {
    constexpr int PADB = (C::V_ROWS - DH) * 128;
    for (int e = tid; e < NS * PADB / 16; e += NT) {
      int st = e / (PADB / 16), o = e % (PADB / 16);
      const unsigned fill = (C::ONES_ROW && o < 8) ? 0x3F803F80u : 0u;   // first padding row: bf16 1.0 in every key column
      *reinterpret_cast<uint4 *>(smem + VRING + st * C::V_BYTES + DH * 128 + o * 16) = make_uint4(fill, fill, fill, fill);
    }
  }

  const int tiles = (kv_rows + TK - 1) / TK;
  const int tps = (tiles + splits - 1) / splits;
  const int t_begin = sp * tps, t_end = min(tiles, (sp + 1) * tps);
  const unsigned char *kh = reinterpret_cast<const unsigned char *>(kbuf + (size_t)h * Lp * DH);
  const bf16_t *vh = vtbuf + (size_t)h * DH * Lp;

  // ---- per-lane source offsets of this wave's load instructions: 32-bit byte offsets from a wave-uniform address, so a
  // load takes its address as scalar base + one vector register (64-bit per-lane pointers cost the 8-wave kernels
  // enough registers to spill, and a spill reload inside the tile loop waits for vmcnt(0), i.e. for the prefetched
  // tiles).  When a wave's instructions are a whole number of swizzle periods apart (LIN: every head size without a
  // K tail) they differ only by a uniform stride and share one offset register per operand.
  constexpr bool LIN = !C::TAIL8 && C::K_INSTR % C::NWL == 0 && C::V_INSTR % C::NWL == 0 &&
                       (C::NWL * 1024) % (16 * C::KROW) == 0;
  unsigned koff[C::LK];      // byte offset inside a K tile
  unsigned char *kdst[C::LK];
#pragma unroll
  for (int i = 0; i < C::LK; ++i) {
    int ins = min(i * C::NWL + (wave & (C::NWL - 1)), C::K_INSTR - 1);   // surplus slots repeat the last instruction (same data)
    int off = ins * 1024 + lane * 16;
    int r = off / C::KROW, p = (off % C::KROW) >> 4;
    koff[i] = (unsigned)(r * C::KROW + ((p ^ C::kkey(r)) << 4));
    kdst[i] = smem + ins * 1024;
  }
  unsigned voff[C::LV];      // byte offset inside the head's V^T (without the tile's column offset): row r < 128, Lp < 2^23 rows
  unsigned char *vdst[C::LV];
#pragma unroll
  for (int i = 0; i < C::LV; ++i) {
    int ins = min(i * C::NWL + (wave & (C::NWL - 1)), C::V_INSTR - 1);
    int r = ins * 8 + (lane >> 3), p = lane & 7;
    voff[i] = ((unsigned)r * (unsigned)Lp + (unsigned)((p ^ ((r >> 1) & 7)) << 3)) * 2u;
    vdst[i] = smem + VRING + ins * 1024;
  }
  // LIN: a wave's instructions share the first one's per-lane offsets and differ by a uniform stride
  const unsigned vstride = (unsigned)C::NWL * 8u * (unsigned)Lp * 2u;   // bytes between a wave's consecutive V^T instructions (LIN)
  const HeadSource ksrc_h(kh), vsrc_h(vh);
  auto issue_k = [&](auto i_c, int stage, int t) __attribute__((always_inline)) {
    constexpr int i = decltype(i_c)::value;
    const unsigned tile_bytes = (unsigned)t * (unsigned)C::K_BYTES;
    if constexpr (LIN) ksrc_h.load16(koff[0], tile_bytes + (unsigned)i * (C::NWL * 1024), kdst[i] + stage * C::K_BYTES);
    else ksrc_h.load16(koff[i], tile_bytes, kdst[i] + stage * C::K_BYTES);
  };
  auto issue_v = [&](auto i_c, int stage, int t) __attribute__((always_inline)) {
    constexpr int i = decltype(i_c)::value;
    const unsigned tile_bytes = (unsigned)t * (TK * 2u);
    if constexpr (LIN) vsrc_h.load16(voff[0], tile_bytes + (unsigned)i * vstride, vdst[i] + stage * C::V_BYTES);
    else vsrc_h.load16(voff[i], tile_bytes, vdst[i] + stage * C::V_BYTES);
  };
  auto issue = [&](int stage, int t) __attribute__((always_inline)) {
    unrolled<C::LK>([&](auto i_c) __attribute__((always_inline)) { issue_k(i_c, stage, t); });
    unrolled<C::LV>([&](auto i_c) __attribute__((always_inline)) { issue_v(i_c, stage, t); });
  };
  // one of this wave's LPS load instructions of tile t (K instructions first, then V^T)
  auto issue_one = [&](auto idx_c, int stage, int t) __attribute__((always_inline)) {
    constexpr int idx = decltype(idx_c)::value;
    if constexpr (idx < C::LK) issue_k(idx_c, stage, t);
    else issue_v(std::integral_constant<int, idx - C::LK>{}, stage, t);
  };
  // The 8-wave kernel spreads the LPS loads of the tile it prefetches over the MFMAs of a step's two matrix phases
  // (half h of the loads inside phase h): issued as one burst behind the barrier they fill the memory pipeline's queue
  // and hold the loading waves - the critical path of a tile - for some 400 cycles before their first MFMA.
  constexpr int LH0 = C::LPS / 2, LH1 = C::LPS - LH0;
  auto spread_load = [&](auto i_c, auto nf_c, auto half_c, int ld_stage, int ld_t) __attribute__((always_inline)) {
    constexpr int i = decltype(i_c)::value, NF = decltype(nf_c)::value, half = decltype(half_c)::value;
    if constexpr (half >= 0) {
      constexpr int LH = half == 0 ? LH0 : LH1;
      constexpr int j = spread_slot(i, NF, LH);
      if constexpr (j >= 0) issue_one(std::integral_constant<int, (half == 0 ? 0 : LH0) + j>{}, ld_stage, ld_t);
    }
  };
  auto burst_half = [&](auto half_c, int ld_stage, int ld_t) __attribute__((always_inline)) {
    constexpr int half = decltype(half_c)::value;
    unrolled<(half == 0 ? LH0 : LH1)>([&](auto j_c) __attribute__((always_inline)) {
      issue_one(std::integral_constant<int, (half == 0 ? 0 : LH0) + decltype(j_c)::value>{}, ld_stage, ld_t);
    });
  };
  // tiles in flight ahead of the one being worked on: NS - 1, or NS - 2 for the 8-wave schedule (see its loop), which
  // always issues NS - 2 tiles (a short split repeats its last tile: its steps count on LPS loads in flight per step)
  const bool loader = wave < C::NWL;
  if constexpr (NW == 8) {
    if (loader && t_begin < t_end) {
#pragma unroll
      for (int i = 0; i < NS - 2; ++i) issue(i, min(t_begin + i, t_end - 1));
    }
  } else {
#pragma unroll
    for (int i = 0; i < NS - 1; ++i)
      if (t_begin + i < t_end) issue(i, t_begin + i);
  }

  // ---- Q fragments (B operand): lane holds query q0 + l32, channels ks*16 + 8*hi .. +7
  bf16x8 qf[C::KS16];
  bf16x4 qtail = {0, 0, 0, 0};
  {
    const int qi = q0 + l32;
    const bf16_t *qp = q + ((size_t)(h / hpi) * nq + qi) * ldq + (size_t)(h % hpi) * DH;
#pragma unroll
    for (int ks = 0; ks < C::KS16; ++ks) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (qi < nq) v = *reinterpret_cast<const uint4 *>(qp + ks * 16 + hi * 8);
      qf[ks] = __builtin_bit_cast(bf16x8, v);
    }
    if constexpr (C::TAIL8) {
      uint2 v = make_uint2(0, 0);
      if (qi < nq) v = *reinterpret_cast<const uint2 *>(qp + C::KS16 * 16 + hi * 4);
      qtail = __builtin_bit_cast(bf16x4, v);
    }
  }

  f32x16 oacc[C::CB];
#pragma unroll
  for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[cb][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;   // running maximum of the raw scores; per-lane partial sum
  const float sl2 = kLog2e / sqrtf((float)DH);
  // PRE: probabilities are taken relative to a reference exponent m_ref per query that only moves on the first tile of
  // a split and when a later score exceeds the largest one seen at the last move by 8 or more (see softmax):
  // p = 2^(s - m_ref).  -m_ref is kept in a 16-register block that seeds the score accumulators (the C operand of a
  // tile's first MFMA), so the subtraction costs no VALU instruction: the softmax of an element is exp2, convert and,
  // where the denominator is not a row of O^T, one addition.
  float m_ref = 0.f;
  f32x16 cneg;
#pragma unroll
  for (int r = 0; r < 16; ++r) cneg[r] = 0.f;

  // fragment addressing, loop invariant: address = row base + ((chunk ^ key) << 4); the chunk's low bit is the
  // half-wave index, so it is folded into the per-lane key and the rest of the chunk index is a compile-time XOR mask
  // Per-lane parts of the LDS addresses, one register per K=16 slice: the row block, the V^T column block and the stage
  // only add constants (a block of 32 rows is a whole number of swizzle periods), which go into the offset field of the
  // LDS reads (where it fits their 16 bits: always with two stages), so a fragment read costs no address arithmetic.
  // Swizzled head sizes: the K = 16 slice only XORs bits 5.. of the address (below the row stride, above the key's low
  // bit), so one register per operand serves every slice.  dh = 72 rows (144 B, no swizzle) keep a register per slice.
  // The 8-wave kernels (two waves per SIMD, one in its matrix phase while the other runs its softmax on the vector unit)
  // spend the registers instead: a v_xor per fragment read is a vector instruction that the matrix phase takes from the
  // partner's softmax (26 per tile at dh = 128).
  constexpr bool XADDR = !C::TAIL8 && NW != 8;
  unsigned kbase[XADDR ? 1 : C::KS16];
#pragma unroll
  for (int ks = 0; ks < (XADDR ? 1 : C::KS16); ++ks)
    kbase[ks] = lds_address(smem) + l32 * C::KROW + ((((hi ^ C::kkey(l32)) << 4)) ^ (ks << 5));
  const unsigned ktail_base = lds_address(smem) + l32 * C::KROW + C::KS16 * 32 + hi * 8;
  unsigned vbase[XADDR ? 1 : 4];
#pragma unroll
  for (int j = 0; j < (XADDR ? 1 : 4); ++j)
    vbase[j] = lds_address(smem) + VRING + l32 * 128 + (((hi ^ ((l32 >> 1) & 7)) << 4) ^ (j << 5));
  // stages past the reach of the reads' 16-bit offset field go through a second base (rings of more than 64 KB)
  const unsigned kbase_hi = kbase[0] + 65536, vbase_hi = vbase[0] + 65536;
  __syncthreads();   // padding rows zeroed (the tile loads in flight do not touch them)

#ifdef PF_TUNING
  unsigned long long ts[24];
#pragma unroll
  for (int i = 0; i < 24; ++i) ts[i] = 0;
  bool tracing = false;
#endif
  bf16x8 pf[2][2];   // P^T fragments of the tile whose PV product comes next
  f32x16 sacc[2];    // S^T of the tile whose softmax comes next (two blocks of 32 kv rows)
  // The K and V^T fragments of the matrix phases are read from LDS PD instructions ahead of the MFMA that uses them
  // (a ring of PD + 1 fragments in registers, the order pinned with scheduling barriers): a wave that is alone in its
  // matrix phase - the other wave of its SIMD being in its softmax - would otherwise wait out an LDS round trip in front
  // of every MFMA.  Five ahead in the 8-wave kernels (three: Flux-scale attention 343.6 -> 340.3 us, long-sequence
  // PixArt 1075 -> 1071 us; two or four ahead measured between).
  constexpr int PD = NW == 8 ? 5 : 3;
  // ---- S^T = K . Q^T for the two 32-row blocks of a tile (K from `stage`); consecutive MFMAs alternate between the blocks
  auto scores = [&](auto stage_c, auto half_c, int ld_stage, int ld_t) __attribute__((always_inline)) {
    constexpr int stage = decltype(stage_c)::value;
    constexpr int NF = 2 * C::KS16;
    auto kread = [&](auto i_c) __attribute__((always_inline)) {
      constexpr int i = decltype(i_c)::value;
      constexpr int off = stage * C::K_BYTES + (i & 1) * 32 * C::KROW;
      if constexpr (XADDR && off > 65535) return lds_read16_async<((i >> 1) << 5), off - 65536>(kbase_hi);
      else if constexpr (XADDR) return lds_read16_async<((i >> 1) << 5), off>(kbase[0]);
      else return lds_read16_async<0, off>(kbase[i >> 1]);
    };
    bf16x8 ring[PD + 1];
    unrolled<PD>([&](auto i_c) __attribute__((always_inline)) { ring[decltype(i_c)::value] = kread(i_c); });
    if constexpr (!PRE) {
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[b2][r] = 0.f;
    }
    unrolled<NF>([&](auto i_c) __attribute__((always_inline)) {
      constexpr int i = decltype(i_c)::value;
      if constexpr (i + PD < NF) {
        ring[(i + PD) % (PD + 1)] = kread(std::integral_constant<int, i + PD>{});
        lds_wait<PD>(ring[i % (PD + 1)]);
      } else {
        lds_wait<NF - 1 - i>(ring[i % (PD + 1)]);
      }
      spread_load(i_c, std::integral_constant<int, NF>{}, half_c, ld_stage, ld_t);
      __builtin_amdgcn_sched_barrier(0);
      constexpr int b2 = i & 1, ks = i >> 1;
      sacc[b2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[i % (PD + 1)], qf[ks], (PRE && ks == 0) ? cneg : sacc[b2], 0, 0, 0);
    });
    if constexpr (C::TAIL8) {
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2) {
        bf16x4 kf4 = *reinterpret_cast<const bf16x4 *>(smem + (ktail_base - lds_address(smem)) + (stage * C::K_BYTES + b2 * 32 * C::KROW));
        sacc[b2] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(__builtin_bit_cast(short4v, kf4),
                                                            __builtin_bit_cast(short4v, qtail), sacc[b2], 0, 0, 0);
      }
    }
  };
  // ---- online softmax of tile t on the raw scores in sacc (the positive scale commutes with max) and its P^T fragments
  auto softmax = [&](int t) __attribute__((always_inline)) {
    if ((t + 1) * TK > kv_rows) {
      const int jbase = t * TK + 4 * hi;
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (jbase + b * 32 + 8 * (r >> 2) + (r & 3) >= kv_rows) sacc[b][r] = -INFINITY;
    }
    // maximum of the tile's scores per query (both lanes of a query agree: the other half-wave's value comes through the
    // vector unit's half-wave swap; an LDS permute would queue behind the fragment reads of all eight waves and cost the
    // wave an LDS round trip per tile)
    auto tile_max = [&]() __attribute__((always_inline)) {
      float m = sacc[0][0];
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) m = fmaxf(m, sacc[b][r]);
      auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(m), __float_as_uint(m), false, false);
      return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
    };
    float psum = 0.f;
    unsigned pk[2][8];   // packed bf16 pairs (r, r+1) of the softmax weights
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    if constexpr (PRE) {
      // The scores arrive relative to the reference (see cneg), so the weights are exp2 of the accumulators as they
      // are, and the tile's maximum is not needed to form them: it is only computed when the reference has to move,
      // which the weights themselves tell.  Heads whose denominator comes out of the matrix pipe keep the reference
      // kRefBias above the largest score seen at its last move and test the exponent's top bit of the packed weights
      // (a weight of 2 or more, an infinity or a NaN sets it; sixteen words OR-ed three at a time); the others test the
      // lane's partial sum, which they form anyway.  Either way the reference moves when a score exceeds the largest one
      // at the last move by 8 or more (up to 13 for the sum test), and on the first tile of a split.
      constexpr float kRefBias = C::ONES_ROW ? 7.f : 0.f;
      constexpr float kSumLimit = 8192.f;
      const bool first = t == t_begin;
      bool move = first;
      for (;;) {
        if (move) {
          const float tmax = tile_max();
          const float delta = first ? tmax + kRefBias : fmaxf(tmax + kRefBias, 0.f);
#pragma unroll
          for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[b][r] -= delta;
          if (!first) {
            const float alpha = __builtin_amdgcn_exp2f(-delta);
            l_run *= alpha;
#pragma unroll
            for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
              for (int r = 0; r < 16; ++r) oacc[cb][r] *= alpha;
          }
          m_ref += delta;
#pragma unroll
          for (int r = 0; r < 16; ++r) cneg[r] = -m_ref;
        }
        psum = 0.f;
        unsigned any = 0;
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int r = 0; r < 16; r += 2) {
            float p0 = __builtin_amdgcn_exp2f(sacc[b][r]);
            float p1 = __builtin_amdgcn_exp2f(sacc[b][r + 1]);
            if constexpr (!C::ONES_ROW) psum += p0 + p1;
            bf16x2 pp = {(bf16_t)p0, (bf16_t)p1};
            pk[b][r >> 1] = __builtin_bit_cast(unsigned, pp);
            if constexpr (C::ONES_ROW) any |= pk[b][r >> 1];
          }
        const bool bad = C::ONES_ROW ? (any & 0x40004000u) != 0 : !(psum < kSumLimit);
        if (move || __builtin_amdgcn_ballot_w64(bad) == 0) break;
        move = true;
      }
      if constexpr (!C::ONES_ROW) l_run += psum;
    } else {
      const float tmax = tile_max();
      const float m_new = fmaxf(m_run, tmax);
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * sl2);
      const float mneg = -m_new * sl2;
      m_run = m_new;
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          float p0 = __builtin_amdgcn_exp2f(fmaf(sacc[b][r], sl2, mneg));
          float p1 = __builtin_amdgcn_exp2f(fmaf(sacc[b][r + 1], sl2, mneg));
          if constexpr (!C::ONES_ROW) psum += p0 + p1;
          bf16x2 pp = {(bf16_t)p0, (bf16_t)p1};
          pk[b][r >> 1] = __builtin_bit_cast(unsigned, pp);
        }
      if constexpr (!C::ONES_ROW) l_run = l_run * alpha + psum;
      if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {   // skip the rescale when no lane's maximum moved
#pragma unroll
        for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[cb][r] *= alpha;
      }
    }
    // ---- O^T += V^T . P^T.  For each K=16 step the half-waves trade registers so that lane-half `hi` holds the
    // weights of kv rows 16*step + 8*hi .. +7 (in order); V^T supplies the same rows with one 16-byte read.
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        auto x0 = __builtin_amdgcn_permlane32_swap(pk[b][4 * s2], pk[b][4 * s2 + 2], false, false);
        auto x1 = __builtin_amdgcn_permlane32_swap(pk[b][4 * s2 + 1], pk[b][4 * s2 + 3], false, false);
        uint4 u = make_uint4(x0[0], x1[0], x0[1], x1[1]);
        pf[b][s2] = __builtin_bit_cast(bf16x8, u);
      }
  };
  // ---- O^T += V^T . P^T with the V^T tile of `stage` and the fragments softmax left; consecutive MFMAs go to different
  // 32-channel blocks of O^T
  auto pv = [&](auto stage_c, auto half_c, int ld_stage, int ld_t) __attribute__((always_inline)) {
    constexpr int stage = decltype(stage_c)::value;
    constexpr int NF = 4 * C::CB;
    auto vread = [&](auto i_c) __attribute__((always_inline)) {
      constexpr int i = decltype(i_c)::value;
      constexpr int off = stage * C::V_BYTES + (i % C::CB) * 32 * 128;
      if constexpr (XADDR && off > 65535) return lds_read16_async<((i / C::CB) << 5), off - 65536>(vbase_hi);
      else if constexpr (XADDR) return lds_read16_async<((i / C::CB) << 5), off>(vbase[0]);
      else return lds_read16_async<0, off>(vbase[i / C::CB]);
    };
    bf16x8 ring[PD + 1];
    unrolled<PD>([&](auto i_c) __attribute__((always_inline)) { ring[decltype(i_c)::value] = vread(i_c); });
    unrolled<NF>([&](auto i_c) __attribute__((always_inline)) {
      constexpr int i = decltype(i_c)::value;
      if constexpr (i + PD < NF) {
        ring[(i + PD) % (PD + 1)] = vread(std::integral_constant<int, i + PD>{});
        lds_wait<PD>(ring[i % (PD + 1)]);
      } else {
        lds_wait<NF - 1 - i>(ring[i % (PD + 1)]);
      }
      spread_load(i_c, std::integral_constant<int, NF>{}, half_c, ld_stage, ld_t);
      __builtin_amdgcn_sched_barrier(0);
      constexpr int j = i / C::CB, cb = i % C::CB;
      oacc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[i % (PD + 1)], pf[j >> 1][j & 1], oacc[cb], 0, 0, 0);
    });
  };
  if constexpr (NW == 4) {
  auto tile_step = [&](int t, auto stage_c) __attribute__((always_inline)) {
    constexpr int stage = decltype(stage_c)::value;
    // tile t has landed once at most min(NS-2, tiles left after t) later tiles of this wave are still in flight
    if (NS >= 4 && t + 2 < t_end) wait_vmcnt<(NS >= 4 ? 2 * C::LPS : 0)>();
    else if (NS >= 3 && t + 1 < t_end) wait_vmcnt<(NS >= 3 ? C::LPS : 0)>();
    else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();         // ... for every wave; and every wave is done with the stage of tile t-1
    asm volatile("" ::: "memory");
    if (t + NS - 1 < t_end) issue((stage + NS - 1) % NS, t + NS - 1);

    scores(stage_c, std::integral_constant<int, -1>{}, 0, 0);
    softmax(t);
    pv(stage_c, std::integral_constant<int, -1>{}, 0, 0);
  };
  for (int t = t_begin; t < t_end; t += NS) {
    tile_step(t, std::integral_constant<int, 0>{});
    if (t + 1 < t_end) tile_step(t + 1, std::integral_constant<int, 1>{});
    if constexpr (NS >= 3) {
      if (t + 2 < t_end) tile_step(t + 2, std::integral_constant<int, 2>{});
    }
    if constexpr (NS >= 4) {
      if (t + 3 < t_end) tile_step(t + 3, std::integral_constant<int, 3>{});
    }
  }
  } else {
    // 8 waves, two per SIMD (waves w and w + 4), one barrier per tile for all of them.  A wave's tile is a matrix phase
    // (PV of the previous tile, then S of this one: 32 MFMAs) and a vector phase (softmax: exponentials, conversions).
    // The two waves of a SIMD run them in opposite order, so that after every barrier one is in its matrix phase while
    // the other is in its vector phase and they swap half a tile later:
    //   waves 0..3:  PV(t-1), S(t)   | softmax(t)
    //   waves 4..7:  softmax(t-1)    | PV(t-1), S(t)
    // Either way the previous tile's V^T stage stays live one step longer, so the prefetch distance is NS - 2 tiles:
    // at step t the loads of tile t + NS - 2 go into the stage tile t - 2 used.
    static_assert(NW == 4 || NS == 4, "the 8-wave schedule is written for a four-stage ring");
    // A wave in its matrix phase asks for issue priority over the wave in its vector phase: an MFMA needs the vector
    // issue port for a few cycles, the arbiter otherwise favours the older wave (waves 0..3) in every conflict, and
    // waves 4..7 then crawl through their MFMAs while waves 0..3 run their softmax and idle at the barrier afterwards.
    // (C4 attention 409 -> 400 us, C5 1310 -> 1275 us; priorities 1, 2 and 3 measure the same)
    constexpr int PRIO_MATRIX = 1;
    const bool late = wave >= 4;
    // (the two schedules are separate loops so that neither pays for the other's live registers)
    // Waves 0..3 load: they wait for their own loads of tile t before the barrier, so that behind the barrier the tile is
    // complete for every wave, and issue the loads of tile t + NS - 2 inside the step's matrix phases.  Waves 4..7 only
    // meet the barrier.
    auto top = [&](int, auto) __attribute__((always_inline)) {
      if (!late) wait_vmcnt<C::LPS>();   // tile t landed; the loads of the step before (tile t + 1 or its stand-in) may be in flight
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
    };
    auto pv_last = [&]() __attribute__((always_inline)) {
      switch ((t_end - 1 - t_begin) % NS) {
        case 0: pv(std::integral_constant<int, 0>{}, std::integral_constant<int, -1>{}, 0, 0); break;
        case 1: pv(std::integral_constant<int, 1>{}, std::integral_constant<int, -1>{}, 0, 0); break;
        case 2: pv(std::integral_constant<int, 2>{}, std::integral_constant<int, -1>{}, 0, 0); break;
        default: pv(std::integral_constant<int, 3 % NS>{}, std::integral_constant<int, -1>{}, 0, 0); break;
      }
    };
    constexpr std::integral_constant<int, 0> S0{};
    constexpr std::integral_constant<int, 1> S1{};
    constexpr std::integral_constant<int, 2> S2{};
    constexpr std::integral_constant<int, 3> S3{};
    constexpr std::true_type FIRST{};
    constexpr std::false_type LATER{};
    // Loop shape, both schedules: the first tile of the split (which has no previous tile to finish) and the up to three
    // steps that bring the ring back to stage 0 stand in front of the loop, the loop body is four steps without a branch
    // out of it, and up to three steps follow it.  With exits between the steps of the body the register allocator
    // placed the O^T accumulators differently in different steps and copied all of them (32 to 40 64-bit moves) once or
    // twice per loop iteration.  (Only the kernels that take prescaled queries - the ones a stage launches - have that
    // shape where it fits: with plain queries the dh = 128 kernel would spill under it and keeps the loop with exits.)
    constexpr bool PEELED = PRE || DH != 128;
    if (!late) {
      auto step = [&](int t, auto stage_c, auto first_c) __attribute__((always_inline)) {
        constexpr int stage = decltype(stage_c)::value;
        PF_STAMP(stage * 6 + 0);
        top(t, stage_c);
        PF_STAMP(stage * 6 + 1);
        __builtin_amdgcn_s_setprio(PRIO_MATRIX);
        // prefetch of tile t + NS - 2 (past the end: the last tile again, into a stage nobody reads any more)
        const int ld_t = min(t + NS - 2, t_end - 1);
        constexpr int ld_stage = (stage + NS - 2) % NS;
        constexpr std::integral_constant<int, 0> h0{};
        constexpr std::integral_constant<int, 1> h1{};
        if constexpr (!decltype(first_c)::value) pv(std::integral_constant<int, (stage + NS - 1) % NS>{}, h0, ld_stage, ld_t);
        else burst_half(h0, ld_stage, ld_t);
        PF_STAMP(stage * 6 + 2);
        scores(stage_c, h1, ld_stage, ld_t);
        PF_STAMP(stage * 6 + 3);
        __builtin_amdgcn_s_setprio(0);
        softmax(t);
        PF_STAMP(stage * 6 + 4);
      };
      if constexpr (!PEELED) {
        for (int t = t_begin; t < t_end; t += NS) {
          if (t > t_begin) step(t, S0, LATER);
          else step(t, S0, FIRST);
          if (t + 1 < t_end) step(t + 1, S1, LATER);
          if (t + 2 < t_end) step(t + 2, S2, LATER);
          if (t + 3 < t_end) step(t + 3, S3, LATER);
        }
      } else if (t_begin < t_end) {
        int t = t_begin;
        step(t, S0, FIRST); ++t;
        if (t < t_end) {
          step(t, S1, LATER); ++t;
          if (t < t_end) {
            step(t, S2, LATER); ++t;
            if (t < t_end) { step(t, S3, LATER); ++t; }
          }
        }
        for (; t + NS <= t_end; t += NS) {
#ifdef PF_TUNING
          tracing = blockIdx.x == 0 && t == t_begin + 8 * NS;
#endif
          step(t, S0, LATER);
          step(t + 1, S1, LATER);
          step(t + 2, S2, LATER);
          step(t + 3, S3, LATER);
        }
#ifdef PF_TUNING
        tracing = false;
#endif
        if (t < t_end) {
          step(t, S0, LATER); ++t;
          if (t < t_end) {
            step(t, S1, LATER); ++t;
            if (t < t_end) step(t, S2, LATER);
          }
        }
      }
      if (t_begin < t_end) {
        pv_last();
      }
    } else {
      auto step = [&](int t, auto stage_c, auto first_c) __attribute__((always_inline)) {
        constexpr int stage = decltype(stage_c)::value;
        PF_STAMP(stage * 6 + 0);
        top(t, stage_c);
        PF_STAMP(stage * 6 + 1);
        if constexpr (!decltype(first_c)::value) {
          softmax(t - 1);
          PF_STAMP(stage * 6 + 2);
          __builtin_amdgcn_s_setprio(PRIO_MATRIX);
          pv(std::integral_constant<int, (stage + NS - 1) % NS>{}, std::integral_constant<int, -1>{}, 0, 0);
        } else {
          __builtin_amdgcn_s_setprio(PRIO_MATRIX);
        }
        PF_STAMP(stage * 6 + 3);
        scores(stage_c, std::integral_constant<int, -1>{}, 0, 0);
        PF_STAMP(stage * 6 + 4);
        __builtin_amdgcn_s_setprio(0);
      };
      if constexpr (!PEELED) {
        for (int t = t_begin; t < t_end; t += NS) {
          if (t > t_begin) step(t, S0, LATER);
          else step(t, S0, FIRST);
          if (t + 1 < t_end) step(t + 1, S1, LATER);
          if (t + 2 < t_end) step(t + 2, S2, LATER);
          if (t + 3 < t_end) step(t + 3, S3, LATER);
        }
      } else if (t_begin < t_end) {
        int t = t_begin;
        step(t, S0, FIRST); ++t;
        if (t < t_end) {
          step(t, S1, LATER); ++t;
          if (t < t_end) {
            step(t, S2, LATER); ++t;
            if (t < t_end) { step(t, S3, LATER); ++t; }
          }
        }
        for (; t + NS <= t_end; t += NS) {
#ifdef PF_TUNING
          tracing = blockIdx.x == 0 && t == t_begin + 8 * NS;
#endif
          step(t, S0, LATER);
          step(t + 1, S1, LATER);
          step(t + 2, S2, LATER);
          step(t + 3, S3, LATER);
        }
#ifdef PF_TUNING
        tracing = false;
#endif
        if (t < t_end) {
          step(t, S0, LATER); ++t;
          if (t < t_end) {
            step(t, S1, LATER); ++t;
            if (t < t_end) step(t, S2, LATER);
          }
        }
      }
      if (t_begin < t_end) {
        softmax(t_end - 1);
        pv_last();
      }
    }
  }
  wait_vmcnt<0>();
#ifdef PF_TUNING
  if (NW == 8 && blockIdx.x == 0 && lane == 0) {
#pragma unroll
    for (int i = 0; i < 24; ++i) g_attn_trace[wave][i] = ts[i];
  }
#endif

  // ---- finish
  // O^T row DH sits in block DH / 32 at local row DH % 32 = 8 * (r / 4) + 4 * hi + r % 4: for DH = 72 that is register 4
  // of the lanes with hi = 0, i.e. lane l32 holds the sum of query l32
  static_assert(!C::ONES_ROW || (DH % 32) == 8, "register index of the ones row is worked out for DH % 32 == 8");
  const float l_tot = C::ONES_ROW ? __shfl(oacc[C::CB - 1][4], l32, kWave) : l_run + __shfl_xor(l_run, 32, kWave);
  const int qi = q0 + l32;
  const int d = H * DH;
  if (splits > 1) {
    // Partial result of this key split: the normalised output row in fp16 (values of the size of V's, 11 bits against
    // the 8 the final bf16 output keeps; half the bytes of fp32 numerators, and this traffic is the combine kernel's
    // whole cost), the reference exponent and the denominator in fp32.  A split that saw no key writes zeros.
    // The rows go through LDS: in registers a lane holds runs of four channels of its query, which stored directly are
    // 8-byte pieces 2 d bytes apart (64 addresses per store instruction; with three rounds of workgroups per launch
    // those stores were 17 us of the Flux-scale launch's 379); staged as [query][channel] rows in the wave's own slice
    // of the ring, which nobody reads any more, they leave as 16-byte pieces of whole rows.
    constexpr int ROWB = DH * 2 + 16;                 // bytes per staged row: 16 more than a row, so that rows start 4 banks apart
    constexpr int CPR = DH * 2 / 16;                  // 16-byte chunks per row
    static_assert(NW * 32 * ROWB <= NS * C::STAGE, "the staged rows of all waves fit the ring");
    __syncthreads();                                  // every wave has read its last fragments
    unsigned char *rows = smem + wave * (32 * ROWB);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        int c = cb * 32 + 8 * g + 4 * hi;
        if (c < DH) {
          f16x4 o4;
#pragma unroll
          for (int e = 0; e < 4; ++e) o4[e] = (_Float16)(oacc[cb][4 * g + e] * inv);
          *reinterpret_cast<f16x4 *>(rows + l32 * ROWB + c * 2) = o4;
        }
      }
    // (the wave reads back only what it wrote itself: program order within the wave is enough)
    _Float16 *op0 = reinterpret_cast<_Float16 *>(ws) + ((size_t)sp * nq + q0) * d + (size_t)h * DH;
#pragma unroll
    for (int it = 0; it < (32 * CPR + 63) / 64; ++it) {
      const int idx = it * 64 + lane, r = idx / CPR, ch = idx - r * CPR;
      if (r < 32 && q0 + r < nq)
        *reinterpret_cast<uint4 *>(op0 + (size_t)r * d + ch * 8) = *reinterpret_cast<const uint4 *>(rows + r * ROWB + ch * 16);
    }
    if (hi == 0 && qi < nq) {
      float *ml = ws + (size_t)splits * nq * d + (((size_t)sp * nq + qi) * H + h) * 2;
      ml[0] = (PRE ? m_ref : m_run * sl2) * kLn2;   // natural-log domain reference of the scaled scores, for the combine kernel
      ml[1] = l_tot;
    }
    return;
  }
  if (qi >= nq) return;
  {
    const float inv = 1.f / l_tot;
    bf16_t *op = out + ((size_t)(h / hpi) * nq + qi) * ldo + (size_t)(h % hpi) * DH;
#pragma unroll
    for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        int c = cb * 32 + 8 * g + 4 * hi;
        if (c < DH) {
          bf16x4 o4;
#pragma unroll
          for (int e = 0; e < 4; ++e) o4[e] = (bf16_t)(oacc[cb][4 * g + e] * inv);
          *reinterpret_cast<bf16x4 *>(op + c) = o4;
        }
      }
  }
}

template <int DH, int NS, bool PRE = false, int NW = 4>
hipError_t launch2(const AttnArgs &a, hipStream_t s) {
  using C = Cfg<DH, NW>;
  constexpr int TQ = C::TQ;
  static_assert(2 * C::LPS <= 63, "two tiles of loads must fit the vmcnt counter");
  constexpr int smem = NS * C::STAGE;
  if (hipError_t e = allow_dynamic_lds<&attn_mfma2_kernel<DH, NS, PRE, NW>, smem>(); e != hipSuccess) return e;
  const int qtiles = (a.nq + TQ - 1) / TQ;
  const int B = a.batch > 1 ? a.batch : 1;
  dim3 g(qtiles * a.n_heads * B * a.splits);
  attn_mfma2_kernel<DH, NS, PRE, NW><<<g, 64 * NW, smem, s>>>((const bf16_t *)a.q, a.ldq, (const bf16_t *)a.kbuf, (const bf16_t *)a.vtbuf,
                                             a.kv_rows, a.rows_padded, a.n_heads * B, (bf16_t *)a.out, a.ldo, a.nq, a.splits,
                                             qtiles, a.ws, a.n_heads);
  return hipGetLastError();
}

}  // namespace

#ifdef PF_TUNING
}  // namespace pf
extern "C" int pf_attn_trace_read(unsigned long long *out) {   // host array of 8 x 24 stamps
  return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(pf::g_attn_trace), sizeof(unsigned long long) * 8 * 24);
}
namespace pf {
#endif

bool attn_mfma2_takes_prescaled_q(int head_dim) {
  return (head_dim == 64 || head_dim == 72 || head_dim == 128) && (g_attn_stages == 0 || g_attn_stages == 2);
}

// Queries per workgroup the bf16 kernel will use for a launch of nq query rows per image (the split heuristic needs it).
int attn_mfma2_qtile(int nq) {
  if (g_attn_stages != 0) return 128;                 // the pinned ring depths exist for the 4-wave kernel only
  return g_attn_wide == 2 || (g_attn_wide == 0 && nq >= 1024) ? 256 : 128;
}

bool attn_partials_half(const AttnArgs &a) {
  return a.dt == DT_BF16 && a.path != PATH_SIMT && g_attn_variant == 0 && attn_mfma2_supported(a);
}

bool attn_mfma2_supported(const AttnArgs &a) {
  // rows_padded < 2^23: the kernel keeps a V^T row offset (up to 127 rows of rows_padded elements) in 32 bits of bytes
  return (a.head_dim == 64 || a.head_dim == 72 || a.head_dim == 128) && a.rows_padded % TK == 0 && a.rows_padded < (1 << 23);
}


hipError_t launch_attn_mfma2(const AttnArgs &a, hipStream_t s) {
  if (a.nq <= 0) return hipSuccess;
  // Two stages by default: in-stage A/B runs on MI355X showed no gain from a third stage for dh = 64 / 72 (1626 vs
  // 1635 us on the 64K-key PixArt stage) and a loss for dh = 128, where it halves the workgroups per CU (430 vs 565 us).
  if (attn_mfma2_qtile(a.nq) == 256) {
    // four stages of 32 KB (dh = 128) are 128 KB of the CU's 160 KB
    if (a.q_prescaled) {
      if (a.head_dim == 64) return launch2<64, 4, true, 8>(a, s);
      if (a.head_dim == 72) return launch2<72, 4, true, 8>(a, s);
      return launch2<128, 4, true, 8>(a, s);
    }
    if (a.head_dim == 64) return launch2<64, 4, false, 8>(a, s);
    if (a.head_dim == 72) return launch2<72, 4, false, 8>(a, s);
    return launch2<128, 4, false, 8>(a, s);
  }
  const int ns = g_attn_stages ? g_attn_stages : 2;
  if (a.q_prescaled && ns != 2) return hipErrorInvalidValue;   // only the two-stage kernels have the variant
  if (a.q_prescaled) {
    if (a.head_dim == 64) return launch2<64, 2, true>(a, s);
    if (a.head_dim == 72) return launch2<72, 2, true>(a, s);
    return launch2<128, 2, true>(a, s);
  }
  if (a.head_dim == 64) return ns == 3 ? launch2<64, 3>(a, s) : launch2<64, 2>(a, s);
  if (a.head_dim == 72) return ns == 3 ? launch2<72, 3>(a, s) : launch2<72, 2>(a, s);
  return ns == 3 ? launch2<128, 3>(a, s) : launch2<128, 2>(a, s);
}

}  // namespace pf
