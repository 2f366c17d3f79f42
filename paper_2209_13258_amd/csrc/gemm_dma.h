// Main GEMM kernel of libosdp: tiles stream from global memory straight into LDS
// (global_load_lds_dwordx4, no staging registers), a ring of LDS stages keeps one or more K
// blocks in flight behind the MFMAs, and operand fragments are double-buffered in registers.
//
// Needs M % BM == 0, N % BN == 0, K % BK == 0; there are no bounds checks.
//
// LDS layouts.  A direct-to-LDS load of one wave deposits lane i's 16 bytes at base + 16*i, so a
// stage is a sequence of 1 KB chunks that cannot be padded; bank conflicts are avoided by
// permuting which 16 bytes of global memory each lane fetches (an XOR swizzle on the source side):
//   K-contiguous operand  [rows][BK]   : 16-byte chunk c of row r is stored at chunk c ^ f(r),
//       f(r) = (r >> 1) & 7 for BK = 64, (r >> 2) & 3 for BK = 32, so that the 16 rows a
//       ds_read_b128 serves per cycle fall into 16 different 16-byte bank groups.
//   MN-contiguous operand [BK][rows]   : 64-byte granule w of k-row k is stored at granule
//       w ^ (k & 3), so that the 4 k-rows one ds_read_b64_tr_b16 group touches are 64 bytes apart.
#pragma once
#include "gemm_common.h"

namespace osdp {
namespace {

typedef __attribute__((address_space(3))) void *lds_void_ptr;
typedef const __attribute__((address_space(1))) void *global_void_ptr;
typedef __attribute__((ext_vector_type(4))) short dma_s16x4;
typedef __attribute__((ext_vector_type(8))) short dma_s16x8;

// One wave-level direct-to-LDS load: lane i's 16 bytes at src land at LDS byte address dst + 16*i
// (dst is wave-uniform and travels in M0).  Written as inline assembly on purpose: the compiler
// then does not know that LDS is written asynchronously and inserts no waits of its own in front
// of the fragment reads; the kernel orders these loads itself with wait_vmcnt + barrier.
__device__ __forceinline__ void dma16(const uint16_t *src, uint32_t dst) {
  const uint32_t m0 = __builtin_amdgcn_readfirstlane(dst);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(m0), "v"(src) : "memory");
}

__device__ __forceinline__ uint32_t lds_address(const void *p) {
  return static_cast<uint32_t>(reinterpret_cast<size_t>((lds_void_ptr)p));
}

// s_waitcnt vmcnt(n) alone (expcnt and lgkmcnt left at their maxima), gfx9 encoding.
template <int n>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(n >= 0 && n < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14));
}

template <bool kKC, int kRows, int kBK, int kWaves>
struct DmaOperand {
  static constexpr int kElems = kRows * kBK;             // one stage
  static constexpr int kLoads = kElems / 512 / kWaves;   // wave-level loads (1 KB each) per wave per stage
  static_assert(kLoads >= 1 && kLoads * kWaves * 512 == kElems, "stage must divide into 1 KB chunks over the waves");
  static constexpr int CPR = kBK / 8, RPL = 64 / CPR;    // K-contiguous: 16-byte chunks per row, rows per load
  static constexpr int VPR = kRows / 8, KPL = 64 / VPR;  // MN-contiguous: 16-byte vectors per k-row, k-rows per load
  static_assert(kBK == 64 || kBK == 32, "BK is 32 or 64");
  static_assert(kKC || (kRows >= 128 && kRows <= 512), "MN-contiguous tiles are 128..512 wide");

  static __device__ __forceinline__ int swz_k(int row) { return CPR == 8 ? ((row >> 1) & 7) : ((row >> 2) & 3); }

  // Element offset, from the tile origin (mn = 0 of the tile, k = k0), of the 16 bytes this lane fetches in
  // its wave's load 0.  Load p of the wave adds p * load_stride(); the swizzle terms do not change with p
  // because a wave's loads are a multiple of 16 rows (4 k-rows) apart.
  static __device__ __forceinline__ int64_t lane_src(int wave, int lane, int64_t ld) {
    if (kKC) {
      const int row = wave * RPL + lane / CPR;
      const int c = (lane % CPR) ^ swz_k(row);
      return static_cast<int64_t>(row) * ld + c * 8;
    } else {
      const int krow = wave * KPL + lane / VPR;
      const int pv = lane % VPR;
      const int lv = (((pv >> 2) ^ (krow & 3)) << 2) | (pv & 3);
      return static_cast<int64_t>(krow) * ld + lv * 8;
    }
  }
  static __device__ __forceinline__ int64_t load_stride(int64_t ld) {
    return static_cast<int64_t>(kWaves) * (kKC ? RPL : KPL) * ld;
  }
  static __device__ __forceinline__ int64_t block_stride(int64_t ld) { return kKC ? kBK : static_cast<int64_t>(kBK) * ld; }

  // Issues this wave's loads of one K block into the stage at LDS byte address `stage` (the operand's area).
  static __device__ __forceinline__ void issue(const uint16_t *src, int64_t lstride, uint32_t stage, int wave) {
#pragma unroll
    for (int p = 0; p < kLoads; ++p) dma16(src + p * lstride, stage + (wave + kWaves * p) * 1024);
  }

  // Fragment of the 32-row block at mn0 for K step kk: lane (l32, g) gets k = 16*kk + 8*g + 0..7 of row mn0 + l32.
  static __device__ __forceinline__ bf16x8 frag(const uint16_t *s, int mn0, int kk, int lane) {
    if (kKC) {
      const int r = mn0 + (lane & 31);
      const int c = (kk * 2 + (lane >> 5)) ^ swz_k(r);
      return *reinterpret_cast<const bf16x8 *>(s + r * kBK + c * 8);
    } else {
      const int i = lane & 15;
      const int krow = kk * 16 + (lane >> 5) * 8 + (i >> 2);
      const int mn = mn0 + ((lane >> 4) & 1) * 16 + (i & 3) * 4;
      const uint16_t *q = s + krow * kRows + (((mn >> 5) ^ (krow & 3)) << 5) + (mn & 31);
      typedef dma_s16x4 __attribute__((address_space(3))) * lds_s16x4;
      const dma_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(q));
      const dma_s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(q + 4 * kRows));
      const dma_s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      return __builtin_bit_cast(bf16x8, both);
    }
  }
};

template <int BM, int BN, int WM, int WN, int BK, int kStages, bool kAK, bool kBK, int kEpi, bool kAccIn>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void gemm_dma_kernel(GemmParams p, int tiles_m, int tiles_n) {
  constexpr int kWaves = (BM / WM) * (BN / WN);
  constexpr int MB = WM / 32, NB = WN / 32, KS = BK / 16;
  using OpA = DmaOperand<kAK, BM, BK, kWaves>;
  using OpB = DmaOperand<kBK, BN, BK, kWaves>;
  constexpr int kStageElems = OpA::kElems + OpB::kElems;
  constexpr int kLoadsPerStage = OpA::kLoads + OpB::kLoads;
  static_assert(kStages >= 2 && kStages <= 4, "2 to 4 LDS stages");
  static_assert((kStages - 2) * kLoadsPerStage < 64, "in-flight loads must fit the vmcnt counter");
  extern __shared__ __attribute__((aligned(1024))) uint16_t smem[];
  __shared__ uint16_t *s_tab[OSDP_MAX_SHARDS];

  const int tid = threadIdx.x;
  if (kEpi == static_cast<int>(Epilogue::kBf16ShardMajor)) {
    if (tid < OSDP_MAX_SHARDS) s_tab[tid] = static_cast<uint16_t *>(p.shards.p[tid]);
  }
  int tm, tn;
  tile_of_block(tiles_m, tiles_n, &tm, &tn);
  const int m0 = tm * BM, n0 = tn * BN;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = (wave / (BN / WN)) * WM, wn = (wave % (BN / WN)) * WN;
  const int l32 = lane & 31, g = lane >> 5;

  const uint16_t *gA = (kAK ? p.A + static_cast<int64_t>(m0) * p.lda : p.A + m0) + OpA::lane_src(wave, lane, p.lda);
  // B may come in two column segments (two staged slices): the tile lies in one of them
  const bool second = p.n_split && n0 >= p.n_split;
  const uint16_t *baseB = second ? p.B2 : p.B;
  const int64_t ldb = second ? p.ldb2 : p.ldb;
  const int nB = second ? n0 - p.n_split : n0;
  const uint16_t *tileB = kBK ? baseB + static_cast<int64_t>(nB) * ldb : baseB + nB;
  const uint16_t *gB = tileB + OpB::lane_src(wave, lane, ldb);
  const int64_t lsA = OpA::load_stride(p.lda), lsB = OpB::load_stride(ldb);
  const int64_t bsA = OpA::block_stride(p.lda), bsB = OpB::block_stride(ldb);
  const int nk = p.K / BK;

  f32x16 acc[MB][NB];
  if (kAccIn) {
    load_acc_tile<MB, NB>(p, acc, m0 + wm, n0 + wn, l32, g);
  } else {
#pragma unroll
    for (int bm = 0; bm < MB; ++bm)
#pragma unroll
      for (int bn = 0; bn < NB; ++bn)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[bm][bn][i] = 0.f;
  }

  // ---- global -> LDS: the LA + LB wave-level loads of one K block, issued in shares ------------------
  constexpr int LA = OpA::kLoads, LB = OpB::kLoads, L = LA + LB;
  // With two stages block it+1 must be complete before the barrier that sits one K step before the end
  // of block it, so its loads are spread over the K steps before that barrier; with more stages they
  // are spread over all K steps.
  constexpr int kIssueSteps = (kStages == 2 && KS > 1) ? KS - 1 : KS;
  int first_seg = p.k_split ? p.k_split / BK : nk;  // K blocks left in the first B segment
  int64_t lsB_cur = lsB, bsB_cur = bsB;
  const uint32_t lds_base = lds_address(smem);
  // loads [first, last) of the block that gA / gB point at, into `stage`; first / last are compile-time
  auto issue_range = [&](int stage, int first, int last) {
    const uint32_t sa = lds_base + stage * (kStageElems * 2);
    const uint32_t sb = sa + OpA::kElems * 2;
#pragma unroll
    for (int i = 0; i < L; ++i) {
      if (i < first || i >= last) continue;
      if (i < LA) dma16(gA + i * lsA, sa + (wave + kWaves * i) * 1024);
      else dma16(gB + (i - LA) * lsB_cur, sb + (wave + kWaves * (i - LA)) * 1024);
    }
    if (last == L) {  // block fully issued: move on
      gA += bsA;
      gB += bsB_cur;
      if (p.k_split && --first_seg == 0) {  // B continues in its second K segment
        gB = (kBK ? p.B2 + static_cast<int64_t>(n0) * p.ldb2 : p.B2 + n0) + OpB::lane_src(wave, lane, p.ldb2);
        lsB_cur = OpB::load_stride(p.ldb2);
        bsB_cur = OpB::block_stride(p.ldb2);
      }
    }
  };

  // Prologue: K blocks 0 .. kStages-2 are put in flight, block 0 is awaited.
#pragma unroll
  for (int s = 0; s < kStages - 1; ++s)
    if (s < nk) issue_range(s, 0, L);
  if (nk >= kStages - 1) wait_vmcnt<(kStages - 2) * L>();
  else wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();

  bf16x8 fa[2][MB], fb[2][NB];
  auto frags = [&](int stage, int kk, int buf) {
    const uint16_t *cA = smem + stage * kStageElems;
    const uint16_t *cB = cA + OpA::kElems;
#pragma unroll
    for (int bm = 0; bm < MB; ++bm) fa[buf][bm] = OpA::frag(cA, wm + bm * 32, kk, lane);
#pragma unroll
    for (int bn = 0; bn < NB; ++bn) fb[buf][bn] = OpB::frag(cB, wn + bn * 32, kk, lane);
  };
  auto mfmas = [&](int buf) {
#pragma unroll
    for (int bm = 0; bm < MB; ++bm)
#pragma unroll
      for (int bn = 0; bn < NB; ++bn) {
        acc[bm][bn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[buf][bn], fa[buf][bm], acc[bm][bn], 0, 0, 0);
      }
  };

  // Steady state.  Per K block `it` (stage cur) and K step kk:
  //   - the fragments of step kk+1 are read from LDS while the MFMAs of step kk run;
  //   - a share of the loads of block it+kStages-1 goes out (stage nxt, freed by the previous barrier);
  //   - after the MFMAs of the step before the last, every wave has all fragments of block it in
  //     registers: block it+1 is awaited and the workgroup barrier is taken there, so that the last
  //     step's MFMAs cover the first fragment reads of block it+1.
  static_assert(KS == 2 || KS == 4, "K block of 32 or 64");
  frags(0, 0, 0);
  int cur = 0, nxt = kStages - 1;
  for (int it = 0; it < nk; ++it) {
    const bool more = it + kStages - 1 < nk;
    const bool follows = it + 1 < nk;
    const int next_stage = (cur + 1 == kStages) ? 0 : cur + 1;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      if (kk + 1 < KS) frags(cur, kk + 1, (kk + 1) & 1);
      else if (follows) frags(next_stage, 0, 0);
      if (more && kk < kIssueSteps) issue_range(nxt, kk * L / kIssueSteps, (kk + 1) * L / kIssueSteps);
      __builtin_amdgcn_sched_barrier(0);
      mfmas(kk & 1);
      __builtin_amdgcn_sched_barrier(0);
      if (kk == KS - 2) {
        // loads issued after the last load of block it+1: the full blocks it+2 .. it+kStages-2 and the
        // shares of block it+kStages-1 issued so far in this iteration
        constexpr int kYounger = (kStages >= 3) ? (kStages - 3) * L + (KS - 1) * L / kIssueSteps : 0;
        if (more) wait_vmcnt<kYounger>();
        else wait_vmcnt<0>();
        __builtin_amdgcn_s_waitcnt((15) | (7 << 4) | (0 << 8) | (3 << 14));  // lgkmcnt(0): this wave's LDS reads are done
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    cur = next_stage;
    nxt = (nxt + 1 == kStages) ? 0 : nxt + 1;
  }

  store_acc_tile<MB, NB, kEpi>(p, acc, m0 + wm, n0 + wn, l32, g, s_tab);
}

}  // namespace
}  // namespace osdp
