// Large-tile GEMM kernel of libosdp: a 256 x 256 output tile per workgroup of four waves, one wave per SIMD,
// each wave owning a 128 x 128 quarter whose 256 fp32 accumulator registers fill the AGPR half of the
// register file.  Against the eight-wave kernel (waves of 64 x 128) every byte read from LDS feeds a third
// more MFMAs (16 fragment reads per 64 MFMAs instead of 12 per 32).
//
// With one wave per SIMD nothing hides a wave's own stalls, so the K loop is one interleaved instruction
// stream: the 64 MFMAs of a K step of 32 carry, in their shadow, the fragment reads of the next K step and the
// global -> LDS loads of a K block further ahead.  LDS holds two K blocks of 64 (64 KB each: A 256 x 64, then
// B 256 x 64).  A wave-level load of a K-contiguous operand covers 128 contiguous bytes of each of 8 rows, whole
// cache lines: with K blocks of 32 the same bytes take twice the requests (64 bytes of each of 16 rows), and the
// stream from L2 into LDS, which on this chip takes about as long as the MFMAs themselves, slows down by 15 %
// (measured on 8192^3, everything else equal).  One workgroup barrier per K block, at the start of its second K
// step: there every wave holds that step's fragments in registers, so block b's slot is free for the loads of
// block b+2, and the loads of block b+1, issued during the previous block's second step, must have landed.
//
// Same MFMA sequence per output element as every other GEMM kernel of the library (K ascending in steps of 32,
// v_mfma_f32_16x16x32_bf16, the same lane -> k map), so the result bits are the same.
//
// Needs M % 256 == 0, N % 256 == 0, K % 64 == 0, K >= 192 (k_split % 64 == 0, n_split % 256 == 0); no bounds checks.
#pragma once
#include <utility>

#include "gemm_common.h"
#include "gemm_dma.h"

namespace osdp {
namespace {

// f(Int<0>{}), f(Int<1>{}), ..., f(Int<N-1>{}): a loop whose index is a compile-time constant in every iteration, so
// that register arrays are never indexed at run time and nothing depends on the optimiser's unrolling.
template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, Is...>) {
  (f(Int<Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
  static_for_impl(static_cast<F &&>(f), std::make_integer_sequence<int, N>{});
}

// The matrix-core step with its accumulator pinned to AGPRs and updated in place.  Written as inline assembly
// because the compiler, left to place 256 accumulator registers itself, keeps moving them between the two halves of
// the register file inside the K loop.  It then no longer sees an MFMA here, so the two hazards it would have
// covered are covered by hand in the kernel: VALU writes of the accumulators before the first step, and VALU reads
// after the last.  For the same reason the K loop below exists once, for every K block alike (no separate code for
// the last blocks): where two copies of it meet, the compiler copies accumulators from the registers one copy chose
// to those the other chose, with VALU moves it does not know to keep clear of the MFMAs.
__device__ __forceinline__ void mma_16x16x32_agpr(f32x4 &c, bf16x8 a_rows, bf16x8 b_cols) {
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(b_cols), "v"(a_rows));
}

// A wave-level direct-to-LDS load that is issued with all lanes off when `on` is 0 (it then moves nothing): the loads
// of K blocks beyond the last, which the uniform K loop below would otherwise fetch for nobody.  All 64 lanes are
// active wherever the kernel calls this, so EXEC is put back to all ones.
// The source is a byte address common to the wave (in scalar registers) plus a 32-bit byte offset per lane: the 16
// loads of a K block then share two lane offsets that never change, and moving on to the next block is scalar
// arithmetic, where per-lane 64-bit pointers cost 32 registers and a vector add each per block.
__device__ __forceinline__ void dma16_if(uint32_t on, uint64_t base, uint32_t lane_off, uint32_t dst) {  // on: 0 or 0xffffffff
  const uint32_t m0 = __builtin_amdgcn_readfirstlane(dst), half = __builtin_amdgcn_readfirstlane(on);
  asm volatile("s_mov_b32 exec_lo, %0\n\ts_mov_b32 exec_hi, %0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\t"
               "global_load_lds_dwordx4 %2, %3\n\ts_mov_b64 exec, -1"
               ::"s"(half), "s"(m0), "v"(lane_off), "s"(base) : "memory");
}

// A 64-bit value that is the same in every lane, as the compiler can see.
__device__ __forceinline__ uint64_t uniform64(uint64_t v) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v));
  const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v >> 32));
  return (static_cast<uint64_t>(hi) << 32) | lo;
}

// One operand's share of a ring slot: 256 rows (or columns) x 64 k, 32 KB, filled by 32 wave-level
// direct-to-LDS loads of 1 KB, eight per wave.
template <bool kKC>
struct W4Operand {
  static constexpr int kRows = 256, kBK = 64, kWaves = 4;
  static constexpr int kElems = kRows * kBK;  // 32 KB
  static constexpr int kLoads = 8;            // per wave and block
  using Base = DmaOperand<kKC, kRows, kBK, kWaves>;
  // 1 KB chunk that load p of wave w fills.  K-contiguous: chunk c = rows 8c .. 8c+7.  MN-contiguous: chunk c =
  // k-rows 2c, 2c+1, with (c & 1) and ((c >> 2) & 1) fixed over a wave's loads (the source swizzle depends on them).
  static __device__ __forceinline__ constexpr int chunk(int w, int p) {
    return kKC ? p * 4 + w : (w & 1) + 2 * (p & 1) + 4 * (w >> 1) + 8 * (p >> 1);
  }
  static __device__ __forceinline__ int64_t lane_src(int w, int lane, int64_t ld) {
    if (kKC) {
      const int row = chunk(w, 0) * 8 + lane / 8;
      const int c = (lane % 8) ^ Base::swz_k(row);
      return static_cast<int64_t>(row) * ld + c * 8;
    } else {
      const int krow = chunk(w, 0) * 2 + lane / 32;
      return static_cast<int64_t>(krow) * ld + (((lane % 32) * 8) ^ Base::swz_mn(krow));
    }
  }
  static __device__ __forceinline__ constexpr int load_rows(int p) {
    return kKC ? (chunk(0, p) - chunk(0, 0)) * 8 : (chunk(0, p) - chunk(0, 0)) * 2;
  }
  static __device__ __forceinline__ int64_t block_stride(int64_t ld) { return kKC ? kBK : static_cast<int64_t>(kBK) * ld; }
  static __device__ __forceinline__ bf16x8 frag(const uint16_t *slot, int mn0, int kk, int lane) { return Base::frag(slot, mn0, kk, lane); }
};

// kCopy: the launch also carries p.job, the gather of a slice that a later launch will read (the forward GEMM of
// slice j gathers slice j+1 into the other staging slot; a dW launch, which needs no weights, gathers the slices of
// the dX pass that follows it).  Every workgroup copies total_vecs / gridDim.x vectors, 256 per K block: one 16-byte
// load and one 16-byte store per lane and block, against that block's 16 KB of operand loads per wave.  A gather
// kernel of its own cannot run beside this kernel, whose four waves hold every register of their SIMDs: on a second
// stream it only takes turns with the tiles, and both get slower.  The carried copy is not free either (the kernel
// is bound by the memory pipe the copy shares: a 64 MiB slice adds 25 us to a 190 us launch, against 28 us as a
// launch of its own); it saves the launch, its gap and every cross-stream event.
template <bool kAK, bool kBKc, int kEpi, bool kAccIn, bool kCopy = false>
__global__ __launch_bounds__(256, 1)
void gemm_w4_kernel(GemmParams p, int tiles_m, int tiles_n) {
  constexpr int BM = 256, BN = 256, WM = 128, WN = 128;
  constexpr int MB = WM / 16, NB = WN / 16;
  using OpA = W4Operand<kAK>;
  using OpB = W4Operand<kBKc>;
  constexpr int kSlotElems = OpA::kElems + OpB::kElems;  // 64 KB
  constexpr int L = OpA::kLoads + OpB::kLoads;           // 16 wave-level loads per wave and block
  extern __shared__ __attribute__((aligned(1024))) uint16_t smem[];
  uint16_t *const *s_tab = nullptr;
  if constexpr (kEpi == static_cast<int>(Epilogue::kBf16ShardMajor)) {
    __shared__ uint16_t *tab[OSDP_MAX_SHARDS];
    if (threadIdx.x < OSDP_MAX_SHARDS) tab[threadIdx.x] = static_cast<uint16_t *>(p.shards.p[threadIdx.x]);
    s_tab = tab;
  }
  const int tid = threadIdx.x;
  // ---- the carried gather: this workgroup's range of vectors, piece i = vectors first + 256 i + tid ----------
  // Lanes beyond the range's end inside its last piece copy the range's last vector again (the same bytes to the
  // same place); K blocks beyond the last piece issue nothing for the copy (one uniform test per hook), which is what
  // keeps a small slice cheap to carry through a long reduction.
  uint64_t copy_first = 0, copy_last = 0;
  uint32_t copy_pieces = 0;
  const uint16_t *const *g_tab = nullptr;
  if constexpr (kCopy) {
    __shared__ const uint16_t *gtab[OSDP_MAX_SHARDS];
    if (tid < OSDP_MAX_SHARDS) gtab[tid] = static_cast<const uint16_t *>(p.job.src.p[tid]);
    g_tab = gtab;  // read after the prologue's barrier
    const uint64_t per_wg = ((p.job.total_vecs + gridDim.x - 1) / gridDim.x + 255) & ~static_cast<uint64_t>(255);
    const uint64_t first = static_cast<uint64_t>(blockIdx.x) * per_wg;
    if (first < p.job.total_vecs) {
      const uint64_t end = first + per_wg < p.job.total_vecs ? first + per_wg : p.job.total_vecs;
      copy_first = first;
      copy_last = end - 1;
      copy_pieces = static_cast<uint32_t>((end - first + 255) / 256);
    }
  }
  // source address of this lane's vector of piece i
  auto copy_src = [&](uint32_t i, uint32_t *v_out) -> const uint4 * {
    uint64_t v = copy_first + static_cast<uint64_t>(i) * 256 + tid;
    v = v < copy_last ? v : copy_last;
    const uint32_t v32 = static_cast<uint32_t>(v);
    const uint32_t rd = v32 / p.job.vecs_per_row, cv = v32 - rd * p.job.vecs_per_row;
    const uint32_t r = p.job.r0 + rd;
    uint32_t s;
    uint64_t off;
    if (p.job.lay.rows_per_shard > 0) {
      s = r / static_cast<uint32_t>(p.job.lay.rows_per_shard);
      off = static_cast<uint64_t>(r - s * p.job.lay.rows_per_shard) * p.job.lay.O + p.job.c0 + cv * 8u;
    } else {
      const uint64_t f = static_cast<uint64_t>(r) * p.job.lay.O + p.job.c0 + cv * 8u;
      s = static_cast<uint32_t>(f / static_cast<uint64_t>(p.job.lay.L));
      off = f - static_cast<uint64_t>(s) * p.job.lay.L;
    }
    *v_out = v32;
    return reinterpret_cast<const uint4 *>(g_tab[s] + off);
  };
  uint4 copy_data = {0u, 0u, 0u, 0u};  // the piece in flight
  uint32_t copy_v = 0;                 // its destination vector
  uint32_t copy_i = 0;                 // its index
  const uint4 *copy_ptr = nullptr;     // source and destination vector of the piece after it
  uint32_t copy_next_v = 0;

  // A launch split along K: the logical ids of one part are consecutive (so an XCD's tiles still share panels),
  // each part runs its own range of k and stores its own fp32 plane.
  int tm, tn;
  int pid = logical_block();
  int K = p.K;
  int64_t k0 = 0;    // first k of this workgroup's part
  int plane_row = 0;  // its plane starts at this row of C (the planes lie one below the other: ldc = N)
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
  const int wm = (wave >> 1) * WM, wn = (wave & 1) * WN;
  const int l16 = lane & 15, q4 = lane >> 4;

  const bool second = p.n_split && n0 >= p.n_split;
  const uint16_t *baseB = second ? p.B2 : p.B;
  const int64_t ldb = second ? p.ldb2 : p.ldb;
  const int nB = second ? n0 - p.n_split : n0;
  // Source of load i of an operand's current K block: byte address blockX + rowX(i), the same for the whole wave,
  // plus this lane's byte offset laneX (all offsets inside a 256-row block are far below 2^32 bytes).
  uint64_t blockA = uniform64(reinterpret_cast<uint64_t>(kAK ? p.A + static_cast<int64_t>(m0) * p.lda + k0 : p.A + m0 + k0 * p.lda));
  uint64_t blockB = uniform64(reinterpret_cast<uint64_t>(kBKc ? baseB + static_cast<int64_t>(nB) * ldb + k0 : baseB + nB + k0 * ldb));
  const uint32_t laneA = static_cast<uint32_t>(OpA::lane_src(wave, lane, p.lda) * 2);
  uint32_t laneB = static_cast<uint32_t>(OpB::lane_src(wave, lane, ldb) * 2);
  auto rowA = [&](int i) { return static_cast<uint64_t>(OpA::load_rows(i)) * static_cast<uint64_t>(p.lda) * 2; };
  int64_t ldb_cur = ldb;
  auto rowB = [&](int i) { return static_cast<uint64_t>(OpB::load_rows(i)) * static_cast<uint64_t>(ldb_cur) * 2; };
  const int64_t stepA = OpA::block_stride(p.lda);
  int64_t stepB = OpB::block_stride(ldb);
  const int nb = K / 64;
  int first_seg = p.k_split ? p.k_split / 64 : nb;

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

  const uint32_t lds_base = lds_address(smem);
  uint32_t dstA[OpA::kLoads], dstB[OpB::kLoads];
#pragma unroll
  for (int i = 0; i < OpA::kLoads; ++i) dstA[i] = OpA::chunk(wave, i) * 1024;
#pragma unroll
  for (int i = 0; i < OpB::kLoads; ++i) dstB[i] = OpA::kElems * 2 + OpB::chunk(wave, i) * 1024;

  uint32_t load_mask = ~0u;  // all lanes while there are K blocks left to load, none afterwards
  auto issue = [&](int slot, auto idx, int64_t advA, int64_t advB) {
    constexpr int i = decltype(idx)::value;
    const uint32_t sb = lds_base + slot * (kSlotElems * 2);
    if constexpr (i < OpA::kLoads) {
      dma16_if(load_mask, blockA + rowA(i), laneA, sb + dstA[i]);
      if constexpr (i == OpA::kLoads - 1) blockA += static_cast<uint64_t>(advA) * 2;  // on to the next K block
    } else {
      constexpr int j = i - OpA::kLoads;
      dma16_if(load_mask, blockB + rowB(j), laneB, sb + dstB[j]);
      if constexpr (j == OpB::kLoads - 1) blockB += static_cast<uint64_t>(advB) * 2;
    }
  };
  auto block_issued = [&]() {
    if (p.k_split && --first_seg == 0) {  // B continues in its second K segment
      blockB = uniform64(reinterpret_cast<uint64_t>(kBKc ? p.B2 + static_cast<int64_t>(n0) * p.ldb2 : p.B2 + n0));
      laneB = static_cast<uint32_t>(OpB::lane_src(wave, lane, p.ldb2) * 2);
      ldb_cur = p.ldb2;
      stepB = OpB::block_stride(p.ldb2);
    }
  };
  bf16x8 fa[2][MB], fb[2][NB];
  asm volatile("s_nop 7");  // accumulator writes (VALU) settle before the first MFMA reads them

  // prologue: blocks 0 and 1 go in flight; block 0 is awaited and the fragments of its first K step read
  static_for<L>([&](auto i) { issue(0, i, stepA, stepB); });
  block_issued();
  static_for<L>([&](auto i) { issue(1, i, stepA, stepB); });
  block_issued();
  wait_vmcnt<L>();
  __builtin_amdgcn_s_barrier();
  if constexpr (kCopy) {  // piece 0 of the carried gather (the barrier has published the shard table)
    copy_ptr = copy_src(0, &copy_v);
    copy_data = load_global16(copy_ptr);
  }
  {
    const uint16_t *sA = smem, *sB = smem + OpA::kElems;
#pragma unroll
    for (int b = 0; b < MB; ++b) fa[0][b] = OpA::frag(sA, wm + b * 16, 0, lane);
#pragma unroll
    for (int b = 0; b < NB; ++b) fb[0][b] = OpB::frag(sB, wn + b * 16, 0, lane);
  }

  // 64 MFMAs of one K step out of fragment set P; in their shadow the 16 fragment reads of the next K step
  // (slot rs, K step rk) into the other set and, when kLoad, the 16 loads of the block two ahead into slot ls.
  auto kstep = [&](auto par, auto load_, const uint16_t *rs, int rk, int ls, int64_t advA, int64_t advB, bool advance) {
    constexpr int P = decltype(par)::value, Q = P ^ 1;
    constexpr bool kLoad = decltype(load_)::value != 0;
    const uint16_t *nA = rs, *nB = rs + OpA::kElems;
    static_for<MB * NB>([&](auto idx) {
      constexpr int i = decltype(idx)::value, bn = i / MB, bm = i % MB;
      mma_16x16x32_agpr(acc[bm][bn], fa[P][bm], fb[P][bn]);
      if constexpr (i % 3 == 1 && i / 3 < MB + NB) {
        constexpr int r = i / 3;
        if constexpr (r < NB) fb[Q][r] = OpB::frag(nB, wn + r * 16, rk, lane);
        else fa[Q][r - NB] = OpA::frag(nA, wm + (r - NB) * 16, rk, lane);
      }
      if constexpr (kLoad && i % 4 == 2) {
        issue(ls, Int<i / 4>{}, advA, advB);
        if (i / 4 == L - 1 && advance) block_issued();
      }
      // carried gather: in the block's first K step the address of the next piece is worked out; in the second,
      // just behind the barrier where every load has landed, the piece in registers goes out and the next comes in
      // (all three behind one uniform test: once the range is copied the remaining K blocks issue nothing for it)
      if constexpr (kCopy && !kLoad && i == 40) {
        if (copy_i + 1 < copy_pieces) copy_ptr = copy_src(copy_i + 1, &copy_next_v);
      }
      if constexpr (kCopy && kLoad && i == 0) {
        if (copy_i < copy_pieces) store_global16(p.job.dst + copy_v, copy_data);
      }
      if constexpr (kCopy && kLoad && i == 1) {
        if (copy_i + 1 < copy_pieces) {
          copy_data = load_global16(copy_ptr);
          copy_v = copy_next_v;
        }
        ++copy_i;
      }
      __builtin_amdgcn_sched_barrier(0);
    });
  };

  // Every block runs the same code: the last two blocks still issue their load instructions (with every lane off,
  // see dma16_if) and the last still reads fragments nobody uses.  The host sends K >= 192.
  int cur = 0;
  int ahead = 2;  // index of the block the source pointers stand at
  for (int b = 0; b < nb; ++b) {
    const uint16_t *sc = smem + cur * kSlotElems, *sn = smem + (cur ^ 1) * kSlotElems;
    // first K step; its shadow reads the second step's fragments of this block
    kstep(Int<0>{}, Int<0>{}, sc, 1, 0, 0, 0, false);
    // block b is now fully in registers or consumed, and block b+1 must be in LDS
    wait_vmcnt<0>();
    __builtin_amdgcn_s_waitcnt((15) | (7 << 4) | (0 << 8) | (3 << 14));  // lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    const bool advance = ahead + 1 < nb;
    load_mask = ahead < nb ? ~0u : 0u;  // this step loads block `ahead`: there is none beyond nb - 1
    kstep(Int<1>{}, Int<1>{}, sn, 0, cur, advance ? stepA : 0, advance ? stepB : 0, advance);
    ahead += 1;
    cur ^= 1;
  }
  wait_vmcnt<0>();  // surplus loads must have landed before the workgroup gives its LDS back
  if constexpr (kCopy) {
    // the piece still in registers, and whatever the K loop was too short for
    if (copy_i < copy_pieces) store_global16(p.job.dst + copy_v, copy_data);
    for (uint32_t i = copy_i + 1; i < copy_pieces; ++i) {
      uint32_t v;
      const uint4 *src = copy_src(i, &v);
      store_global16(p.job.dst + v, load_global16(src));
    }
  }

  asm volatile("s_nop 15");
  asm volatile("s_nop 15");
  store_acc_tile<MB, NB, kEpi>(p, acc, plane_row + m0 + wm, n0 + wn, l16, q4, s_tab);
}

}  // namespace
}  // namespace osdp
