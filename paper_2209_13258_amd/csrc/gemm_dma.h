// Main GEMM kernel of libosdp: tiles stream from global memory straight into LDS
// (global_load_lds_dwordx4, no staging registers), a ring of LDS stages keeps one or more K
// blocks in flight behind the MFMAs (v_mfma_f32_16x16x32_bf16), and operand fragments are
// double-buffered in registers.
//
// Needs M % BM == 0, N % BN == 0, K % BK == 0; there are no bounds checks.
//
// LDS layouts.  A direct-to-LDS load of one wave deposits lane i's 16 bytes at base + 16*i, so a
// stage is a sequence of 1 KB chunks that cannot be padded; bank conflicts are avoided by
// permuting which 16 bytes of global memory each lane fetches (an XOR swizzle on the source side):
//   K-contiguous operand  [rows][BK]   : 16-byte chunk c of row r is stored at chunk c ^ f(r),
//       f(r) = (r >> 1) & 7 for BK = 64, 2 * ((r >> 3) & 1) for BK = 32, so that the 16 lanes a
//       ds_read_b128 serves per cycle fall into 16 different 16-byte bank groups.
//   MN-contiguous operand [BK][rows]   : 64-byte granule w of k-row k is stored at granule
//       w ^ (k & 3) and its 32-byte halves are swapped when bit 3 of k is set, so that the k-rows the
//       lane groups of one ds_read_b64_tr_b16 phase touch fall into different bank groups.
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

  // A ds_read_b128 is served 16 lanes at a time, and not 16 consecutive ones: measured on the box, lane 0 shares
  // its cycle with lanes 1-3, 12-15 and 20-27 (within each half of the wave the two groups are the lanes with even
  // and with odd parity of lane bits 2, 3 and 4).  With lane = 16 * q + row the swizzles below put the 16 reads
  // of every such group into 16 different 16-byte bank groups.
  static __device__ __forceinline__ int swz_k(int row) { return CPR == 8 ? ((row >> 1) & 7) : (((row >> 3) & 1) << 1); }
  // MN-contiguous: element offset mn of k-row k is stored at mn ^ swz_mn(k): the 64-byte granule index is
  // XORed with k & 3 and the 32-byte half inside the granule with bit 3 of k, so that the 8 k-rows the two
  // lane groups of one transposing-read phase touch (k, k+1, k+2, k+3 and the same + 8) fall into 8 different
  // 32-byte bank groups.
  static __device__ __forceinline__ int swz_mn(int krow) { return ((krow & 3) << 5) | (((krow >> 3) & 1) << 4); }

  // Element offset, from the tile origin (mn = 0 of the tile, k = k0), of the 16 bytes this lane fetches in
  // its wave's load 0.  Load p of the wave adds p * load_stride(); the swizzle terms do not change with p
  // because a wave's loads are a multiple of 16 rows (16 k-rows) apart.
  static __device__ __forceinline__ int64_t lane_src(int wave, int lane, int64_t ld) {
    static_assert(kKC || (kWaves * KPL) % 16 == 0, "a wave's loads must be a multiple of 16 k-rows apart");
    if (kKC) {
      const int row = wave * RPL + lane / CPR;
      const int c = (lane % CPR) ^ swz_k(row);
      return static_cast<int64_t>(row) * ld + c * 8;
    } else {
      const int krow = wave * KPL + lane / VPR;
      const int pv = lane % VPR;
      return static_cast<int64_t>(krow) * ld + ((pv * 8) ^ swz_mn(krow));
    }
  }
  static __device__ __forceinline__ int64_t load_stride(int64_t ld) {
    return static_cast<int64_t>(kWaves) * (kKC ? RPL : KPL) * ld;
  }
  static __device__ __forceinline__ int64_t block_stride(int64_t ld) { return kKC ? kBK : static_cast<int64_t>(kBK) * ld; }

  // Fragment of the 16-row block at mn0 for K step kk (32 wide): lane (l16, q) gets k = 32*kk + 8*q + 0..7 of
  // row mn0 + l16.
  static __device__ __forceinline__ bf16x8 frag(const uint16_t *s, int mn0, int kk, int lane) {
    if (kKC) {
      const int r = mn0 + (lane & 15);
      const int c = (kk * 4 + (lane >> 4)) ^ swz_k(r);
      return *reinterpret_cast<const bf16x8 *>(s + r * kBK + c * 8);
    } else {
      // ds_read_b64_tr_b16: within 16 lanes, lane s supplies 4 consecutive mn of k-row s / 4 and lane i
      // receives the 4 k of mn i; two reads, 4 k-rows apart, give the lane its 8 consecutive k
      const int i = lane & 15;
      const int krow = kk * 32 + (lane >> 4) * 8 + (i >> 2);
      const int mn = mn0 + (i & 3) * 4;
      const uint16_t *q = s + krow * kRows + (mn ^ swz_mn(krow));
      typedef dma_s16x4 __attribute__((address_space(3))) * lds_s16x4;
      const dma_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(q));
      const dma_s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(q + 4 * kRows));
      const dma_s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      return __builtin_bit_cast(bf16x8, both);
    }
  }
};

// Compile-time integers as lambda arguments.
template <int v>
struct Int {
  static constexpr int value = v;
};

// Workgroups of one tile shape that fit a CU's 160 KB of LDS together (at most 2 are aimed for), and the waves
// per SIMD that this takes: the register budget the compiler is held to.
constexpr int dma_groups_per_cu(int BM, int BN, int BK, int kStages) {
  return (2 * (kStages * (BM + BN) * BK * 2 + OSDP_MAX_SHARDS * 8) <= 160 * 1024) ? 2 : 1;
}

template <int BM, int BN, int WM, int WN, int BK, int kStages, bool kAK, bool kBK, int kEpi, bool kAccIn>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64, dma_groups_per_cu(BM, BN, BK, kStages) * (BM / WM) * (BN / WN) / 4)
void gemm_dma_kernel(GemmParams p, int tiles_m, int tiles_n) {
  constexpr int kWaves = (BM / WM) * (BN / WN);
  constexpr int MB = WM / 16, NB = WN / 16, NH = NB / 2;  // 16 x 16 blocks of the wave tile; B blocks per half
  constexpr int KS = BK / 32;                              // K steps per block
  constexpr int U = 2 * KS;                                // micro-steps per block: (K step, half of the B blocks)
  static_assert(NB % 2 == 0, "the wave tile is split in two column halves");
  using OpA = DmaOperand<kAK, BM, BK, kWaves>;
  using OpB = DmaOperand<kBK, BN, BK, kWaves>;
  constexpr int kStageElems = OpA::kElems + OpB::kElems;
  static_assert(kStages >= 2 && kStages <= 4, "2 to 4 LDS stages");
  extern __shared__ __attribute__((aligned(1024))) uint16_t smem[];
  __shared__ uint16_t *s_tab[OSDP_MAX_SHARDS];

  const int tid = threadIdx.x;
  if (kEpi == static_cast<int>(Epilogue::kBf16ShardMajor)) {
    if (tid < OSDP_MAX_SHARDS) s_tab[tid] = static_cast<uint16_t *>(p.shards.p[tid]);
  }
  // A launch split along K: the logical ids of one part are consecutive, each part runs its own range of k and
  // stores its own fp32 plane (the planes lie one below the other: ldc = N).
  int tm, tn;
  int pid = logical_block();
  int K = p.K, plane_row = 0;
  int64_t k0 = 0;
  if (p.k_parts > 1) {
    const int tiles = tiles_m * tiles_n, part = pid / tiles;
    pid -= part * tiles;
    K = p.K / p.k_parts;
    k0 = static_cast<int64_t>(part) * K;
    plane_row = part * p.M;
  }
  tile_of_pid(pid, tiles_m, tiles_n, &tm, &tn);
  const int m0 = tm * BM, n0 = tn * BN;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = (wave / (BN / WN)) * WM, wn = (wave % (BN / WN)) * WN;
  const int l16 = lane & 15, q4 = lane >> 4;

  const uint16_t *gA = (kAK ? p.A + static_cast<int64_t>(m0) * p.lda + k0 : p.A + m0 + k0 * p.lda) + OpA::lane_src(wave, lane, p.lda);
  // B may come in two column segments (two staged slices): the tile lies in one of them
  const bool second = p.n_split && n0 >= p.n_split;
  const uint16_t *baseB = second ? p.B2 : p.B;
  const int64_t ldb = second ? p.ldb2 : p.ldb;
  const int nB = second ? n0 - p.n_split : n0;
  const uint16_t *tileB = kBK ? baseB + static_cast<int64_t>(nB) * ldb + k0 : baseB + nB + k0 * ldb;
  const uint16_t *gB = tileB + OpB::lane_src(wave, lane, ldb);
  const int64_t lsA = OpA::load_stride(p.lda), lsB = OpB::load_stride(ldb);
  const int64_t bsA = OpA::block_stride(p.lda), bsB = OpB::block_stride(ldb);
  const int nk = K / BK;

  f32x4 acc[MB][NB];
  if (kAccIn) {
    load_acc_tile<MB, NB>(p, acc, m0 + wm, n0 + wn, l16, q4);
  } else {
#pragma unroll
    for (int bm = 0; bm < MB; ++bm)
#pragma unroll
      for (int bn = 0; bn < NB; ++bn)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[bm][bn][i] = 0.f;
  }

  // ---- global -> LDS: the LA + LB wave-level loads of one K block, issued in shares ------------------
  constexpr int LA = OpA::kLoads, LB = OpB::kLoads, L = LA + LB;
  static_assert((kStages - 1) * L < 64, "in-flight loads must fit the vmcnt counter");
  // The workgroup barrier of block it sits after the MFMAs of its micro-step U-2 and block it+1 must have
  // landed there.  With two stages the loads of block it+1 can only start once the barrier of block it-1 has
  // freed their stage, so they are spread over the micro-steps before the barrier; with more stages the loads
  // of block it+kStages-1 are spread over all micro-steps.
  constexpr int kIssueSteps = (kStages == 2 && U > 1) ? U - 1 : U;
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

  // Fragments in registers: the A blocks of two K steps (alternating), the B blocks of two micro-steps.
  bf16x8 fa[2][MB], fb[2][NH];
  auto read_a = [&](int stage, int kk, auto buf) {
    const uint16_t *cA = smem + stage * kStageElems;
#pragma unroll
    for (int bm = 0; bm < MB; ++bm) fa[decltype(buf)::value][bm] = OpA::frag(cA, wm + bm * 16, kk, lane);
  };
  auto read_b = [&](int stage, int kk, int half, auto buf) {
    const uint16_t *cB = smem + stage * kStageElems + OpA::kElems;
#pragma unroll
    for (int bn = 0; bn < NH; ++bn) fb[decltype(buf)::value][bn] = OpB::frag(cB, wn + (half * NH + bn) * 16, kk, lane);
  };
  auto mfmas = [&](auto abuf, auto bbuf, auto half) {
#pragma unroll
    for (int bn = 0; bn < NH; ++bn)
#pragma unroll
      for (int bm = 0; bm < MB; ++bm)
        acc[bm][decltype(half)::value * NH + bn] =
            mma_16x16x32(fa[decltype(abuf)::value][bm], fb[decltype(bbuf)::value][bn], acc[bm][decltype(half)::value * NH + bn]);
  };

  // Steady state, one K block `it` (stage cur) = U micro-steps.  In micro-step u = (K step kk, column half h):
  //   - the fragments of micro-step u+1 are read from LDS (the other half of the B blocks; the A blocks too when
  //     it starts a new K step) while the MB * NH MFMAs of micro-step u run;
  //   - a share of the loads of block it+kStages-1 goes out (stage nxt, freed by the previous barrier);
  //   - after the MFMAs of micro-step U-2 every fragment read of block it has been issued: block it+1 is awaited
  //     and the workgroup barrier taken there, so that the last micro-step's MFMAs cover the first fragment
  //     reads of block it+1.
  // `par` is the parity of the block's first K step: A fragments of K step kk sit in fa[(par + kk) & 1].
  int cur = 0, nxt = kStages - 1;
  auto block = [&](int it, auto par) {
    constexpr int P = decltype(par)::value;
    const bool more = it + kStages - 1 < nk;
    const bool follows = it + 1 < nk;
    const int next_stage = (cur + 1 == kStages) ? 0 : cur + 1;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int kk = u >> 1, h = u & 1;
      // fragments of micro-step u+1 (its B half goes to fb[(u+1) & 1]; U is even, so the first micro-step of a
      // block always uses fb[0])
      if (u + 1 < U) {
        const int kk2 = (u + 1) >> 1, h2 = (u + 1) & 1;
        if (h2 == 0) {
          if (((P + kk2) & 1) == 0) read_a(cur, kk2, Int<0>{}); else read_a(cur, kk2, Int<1>{});
        }
        if (((u + 1) & 1) == 0) read_b(cur, kk2, h2, Int<0>{}); else read_b(cur, kk2, h2, Int<1>{});
      } else if (follows) {
        if (((P + KS) & 1) == 0) read_a(next_stage, 0, Int<0>{}); else read_a(next_stage, 0, Int<1>{});
        read_b(next_stage, 0, 0, Int<0>{});
      }
      if (more && u < kIssueSteps) issue_range(nxt, u * L / kIssueSteps, (u + 1) * L / kIssueSteps);
      __builtin_amdgcn_sched_barrier(0);
      if (((P + kk) & 1) == 0) {
        if (h == 0) mfmas(Int<0>{}, Int<0>{}, Int<0>{}); else mfmas(Int<0>{}, Int<1>{}, Int<1>{});
      } else {
        if (h == 0) mfmas(Int<1>{}, Int<0>{}, Int<0>{}); else mfmas(Int<1>{}, Int<1>{}, Int<1>{});
      }
      __builtin_amdgcn_sched_barrier(0);
      if (u == U - 2) {
        // loads issued after the last load of block it+1: the full blocks it+2 .. it+kStages-2 and the
        // shares of block it+kStages-1 issued so far in this block
        constexpr int kYounger = (kStages >= 3) ? (kStages - 3) * L + (U - 1) * L / kIssueSteps : 0;
        if (more) wait_vmcnt<kYounger>();
        else wait_vmcnt<0>();
        __builtin_amdgcn_s_waitcnt((15) | (7 << 4) | (0 << 8) | (3 << 14));  // lgkmcnt(0): this wave's LDS reads are done
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    cur = next_stage;
    nxt = (nxt + 1 == kStages) ? 0 : nxt + 1;
  };

  read_a(0, 0, Int<0>{});
  read_b(0, 0, 0, Int<0>{});
  if (KS % 2 == 0) {
    for (int it = 0; it < nk; ++it) block(it, Int<0>{});
  } else {  // an odd number of K steps per block: the A fragment buffers swap roles from block to block
    for (int it = 0; it < nk; it += 2) {
      block(it, Int<0>{});
      if (it + 1 < nk) block(it + 1, Int<1>{});
    }
  }

  store_acc_tile<MB, NB, kEpi>(p, acc, plane_row + m0 + wm, n0 + wn, l16, q4, s_tab);
}

}  // namespace
}  // namespace osdp
