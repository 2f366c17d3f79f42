// The four-wave 256 x 256 GEMM kernel of gemm_w4.h as a persistent kernel: one workgroup per CU walks through the
// tiles t = w, w + G, w + 2G, ... (G workgroups) and treats their K blocks as one stream.
//
// Why: with one workgroup per CU nothing overlaps a tile's start-up and wind-down with another tile's MFMAs.  A
// tile of the plain kernel pays about 10 us beyond its K loop (the workgroup's launch, the latency of its first two
// K blocks, the drain of its stores): 17 % of a tile with K = 2048, 9 % with K = 4096.  Here the loads run two K
// blocks ahead of the MFMAs across tile boundaries, so the first blocks of the next tile are in LDS before the last
// MFMA of the current one; between the two tiles stand only the stores of the finished tile and the reset of the
// accumulators.  (The stores of tile t are older than the loads of block 2 of tile t+1 in the wave's memory
// counter, which counts loads and stores together and in order: the wait for that block also waits for their
// acknowledgement.)
//
// Same tiles in the same order per XCD, same MFMA sequence per output element as every other GEMM kernel of the
// library: same bits.  Takes what the plain kernel takes except a carried gather: M % 256 == 0, N % 256 == 0
// (n_split % 256 == 0), K % 64 == 0 (k_split % 64 == 0), K >= 192 (per part, when the launch runs parts of the reduction).
#pragma once
#include "gemm_w4.h"

namespace osdp {
namespace {

// Starting a tile's accumulators inside the loop over tiles.  To the compiler an assignment (acc = 0, acc = loaded
// values) would be a new value that has to be merged with the one the K loop carries, and it merges 256 pinned
// registers through scratch memory.  So the reset is itself a matrix-core step on the same registers, c = 0 * 0 + 0,
// written like the K loop's own steps as an update in place ...
__device__ __forceinline__ void acc_clear(f32x4 &c, bf16x8 zero) {
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %1, 0" : "+a"(c) : "v"(zero));
}
// ... and initial values come from memory straight into the accumulator registers; the caller waits (vmcnt) before
// the first MFMA.
__device__ __forceinline__ void acc_load(f32x4 &c, const float *src) {
  asm volatile("global_load_dwordx4 %0, %1, off" : "+a"(c) : "v"(src) : "memory");
}

// The four values of an accumulator block, read where this stands and nowhere else: read by the compiler's own
// copies they may move to the head of the epilogue, all 256 at once, into registers the K loop's fragments hold.
__device__ __forceinline__ f32x4 acc_read(const f32x4 &c) {
  float x0, x1, x2, x3;
  asm volatile("v_accvgpr_read_b32 %0, %4\n\tv_accvgpr_read_b32 %1, %5\n\tv_accvgpr_read_b32 %2, %6\n\tv_accvgpr_read_b32 %3, %7"
               : "=v"(x0), "=v"(x1), "=v"(x2), "=v"(x3) : "a"(c[0]), "a"(c[1]), "a"(c[2]), "a"(c[3]));
  return f32x4{x0, x1, x2, x3};
}

template <bool kAK, bool kBKc, int kEpi, bool kAccIn>
__global__ __launch_bounds__(256, 1)
void gemm_w4p_kernel(GemmParams p, int tiles_m, int tiles_n) {
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
    s_tab = tab;  // read after the prologue's barrier
  }
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = (wave >> 1) * WM, wn = (wave & 1) * WN;
  const int l16 = lane & 15, q4 = lane >> 4;
  // A launch split along K: the tiles of part 0 come first, then those of part 1, ...; each part runs its own range
  // of k and stores its own fp32 plane (the planes lie one below the other in C).
  const int parts = p.k_parts > 1 ? p.k_parts : 1;
  const int part_tiles = tiles_m * tiles_n, tiles = part_tiles * parts, G = gridDim.x;
  const int first = logical_block();  // < tiles: the host launches at most one workgroup per tile
  const int part_k = p.K / parts;
  const int nb = part_k / 64;
  const int my_tiles = (tiles - first + G - 1) / G;

  // ---- the load side: tile `lt`, its next block `lb`, the sources of that block ---------------------------
  int lt = first, lb = 0;
  uint64_t blockA = 0, blockB = 0;
  uint32_t laneB = 0;
  int64_t ldb_cur = p.ldb;
  const uint32_t laneA = static_cast<uint32_t>(OpA::lane_src(wave, lane, p.lda) * 2);
  const int64_t stepA = OpA::block_stride(p.lda);
  int64_t stepB = 0;
  auto rowA = [&](int i) { return static_cast<uint64_t>(OpA::load_rows(i)) * static_cast<uint64_t>(p.lda) * 2; };
  auto rowB = [&](int i) { return static_cast<uint64_t>(OpB::load_rows(i)) * static_cast<uint64_t>(ldb_cur) * 2; };
  int n0l = 0;  // first column of the tile being loaded
  const int seg_blocks = p.k_split / 64;  // K blocks of B's first segment when B has two (0: one segment)
  auto load_tile = [&](int t) {  // point the sources at block 0 of tile t
    int tm, tn;
    const int part = t / part_tiles;
    tile_of_pid(t - part * part_tiles, tiles_m, tiles_n, &tm, &tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const int64_t k0 = static_cast<int64_t>(part) * part_k;
    n0l = n0;
    const bool second = p.n_split && n0 >= p.n_split;
    const uint16_t *baseB = second ? p.B2 : p.B;
    const int nB = second ? n0 - p.n_split : n0;
    ldb_cur = second ? p.ldb2 : p.ldb;
    blockA = uniform64(reinterpret_cast<uint64_t>(kAK ? p.A + static_cast<int64_t>(m0) * p.lda + k0 : p.A + m0 + k0 * p.lda));
    blockB = uniform64(reinterpret_cast<uint64_t>(kBKc ? baseB + static_cast<int64_t>(nB) * ldb_cur + k0 : baseB + nB + k0 * ldb_cur));
    laneB = static_cast<uint32_t>(OpB::lane_src(wave, lane, ldb_cur) * 2);
    stepB = OpB::block_stride(ldb_cur);
  };
  uint32_t load_mask = ~0u;  // all lanes while there are K blocks left to load, none afterwards
  auto block_issued = [&]() {  // after the last load of a block: on to the next block, of this tile or the next
    if (++lb == nb) {
      lb = 0;
      lt += G;
      if (lt < tiles) load_tile(lt);
      else load_mask = 0u;
    } else {
      blockA += static_cast<uint64_t>(stepA) * 2;
      if (lb == seg_blocks) {  // B continues in its second K segment
        ldb_cur = p.ldb2;
        blockB = uniform64(reinterpret_cast<uint64_t>(kBKc ? p.B2 + static_cast<int64_t>(n0l) * ldb_cur : p.B2 + n0l));
        laneB = static_cast<uint32_t>(OpB::lane_src(wave, lane, ldb_cur) * 2);
        stepB = OpB::block_stride(ldb_cur);
      } else {
        blockB += static_cast<uint64_t>(stepB) * 2;
      }
    }
  };

  const uint32_t lds_base = lds_address(smem);
  uint32_t dstA[OpA::kLoads], dstB[OpB::kLoads];
#pragma unroll
  for (int i = 0; i < OpA::kLoads; ++i) dstA[i] = OpA::chunk(wave, i) * 1024;
#pragma unroll
  for (int i = 0; i < OpB::kLoads; ++i) dstB[i] = OpA::kElems * 2 + OpB::chunk(wave, i) * 1024;
  auto issue = [&](int slot, auto idx) {
    constexpr int i = decltype(idx)::value;
    const uint32_t sb = lds_base + slot * (kSlotElems * 2);
    if constexpr (i < OpA::kLoads) dma16_if(load_mask, blockA + rowA(i), laneA, sb + dstA[i]);
    else dma16_if(load_mask, blockB + rowB(i - OpA::kLoads), laneB, sb + dstB[i - OpA::kLoads]);
  };

  // ---- the compute side: tile `ct`, its origin, its accumulators --------------------------------------------
  int ct = first, cb = 0, m0c = 0, n0c = 0;
  f32x4 acc[MB][NB];
#pragma unroll
  for (int bm = 0; bm < MB; ++bm)
#pragma unroll
    for (int bn = 0; bn < NB; ++bn)
      asm volatile("" : "=a"(acc[bm][bn]));  // (a value to the compiler, no instruction: begin_tile sets the registers)
  bf16x8 zero;
#pragma unroll
  for (int i = 0; i < 8; ++i) zero[i] = static_cast<__bf16>(0.0f);
  // Written once, here: an MFMA may not read a register in the two cycles after a VALU instruction wrote it, and the
  // compiler, which does not see the MFMAs inside the asm statements, would otherwise write these zeros anew right
  // in front of each use.
  asm volatile("s_nop 1" : "+v"(zero));
  auto begin_tile = [&](int t, int l16e, int q4e) {
    int tm, tn;
    const int part = t / part_tiles;
    tile_of_pid(t - part * part_tiles, tiles_m, tiles_n, &tm, &tn);
    m0c = tm * BM + part * p.M;  // (row of C: the part's plane starts at row part * M)
    n0c = tn * BN;
    static_for<MB * NB>([&](auto idx) {
      constexpr int i = decltype(idx)::value, bn = i / MB, bm = i % MB;  // the order of the K loop's steps
      if constexpr (kAccIn) {
        const float *src = p.acc_in + static_cast<int64_t>(m0c + wm + bm * 16 + l16e) * p.ld_acc + n0c + wn + bn * 16 + 4 * q4e;
        acc_load(acc[bm][bn], src);
      } else {
        acc_clear(acc[bm][bn], zero);
      }
    });
    if constexpr (kAccIn) wait_vmcnt<0>();
  };

  // prologue: blocks 0 and 1 of the first tile go in flight; block 0 is awaited and its first fragments read
  load_tile(lt);
  static_for<L>([&](auto i) { issue(0, i); });
  block_issued();
  static_for<L>([&](auto i) { issue(1, i); });
  block_issued();
  begin_tile(ct, l16, q4);
  wait_vmcnt<L>();
  __builtin_amdgcn_s_barrier();
  bf16x8 fa[2][MB], fb[2][NB];
  {
    const uint16_t *sA = smem, *sB = smem + OpA::kElems;
#pragma unroll
    for (int b = 0; b < MB; ++b) fa[0][b] = OpA::frag(sA, wm + b * 16, 0, lane);
#pragma unroll
    for (int b = 0; b < NB; ++b) fb[0][b] = OpB::frag(sB, wn + b * 16, 0, lane);
  }

  // 64 MFMAs of one K step out of fragment set P; between them the 16 fragment reads of the next K step (slot rs,
  // K step rk) into the other set and, when kLoad, the 16 loads of the block two ahead into slot ls.
  auto kstep = [&](auto par, auto load_, const uint16_t *rs, int rk, int ls) {
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
        issue(ls, Int<i / 4>{});
        if constexpr (i / 4 == L - 1) block_issued();
      }
      __builtin_amdgcn_sched_barrier(0);
    });
  };

  // One loop over all K blocks of all tiles of this workgroup; every block runs the same code.  Loads beyond the
  // last block of the last tile are issued with every lane off, and the fragments read ahead at the very end
  // are nobody's.
  int cur = 0;
  const int total = my_tiles * nb;
  for (int g = 0; g < total; ++g) {
    const uint16_t *sc = smem + cur * kSlotElems, *sn = smem + (cur ^ 1) * kSlotElems;
    kstep(Int<0>{}, Int<0>{}, sc, 1, 0);
    // this block is now fully in registers or consumed, and the next one must be in LDS
    wait_vmcnt<0>();
    __builtin_amdgcn_s_waitcnt((15) | (7 << 4) | (0 << 8) | (3 << 14));  // lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    kstep(Int<1>{}, Int<1>{}, sn, 0, cur);
    cur ^= 1;
    if (++cb == nb) {  // the tile is complete: store it and start the next (its first blocks are in LDS or on their way)
      cb = 0;
      asm volatile("s_nop 15");
      asm volatile("s_nop 15");
      // The lane's coordinates pass through an empty asm so that every address of the epilogue is computed here:
      // computed ahead of the loop they would sit in registers that the K loop has no room for.
      int l16e = l16, q4e = q4;
      asm volatile("" : "+v"(l16e), "+v"(q4e));
      // one 16 x 16 block at a time (a scheduling fence after each): read all at once, the 256 values would push
      // the K loop's fragments out of their registers
      static_for<MB * NB>([&](auto idx) {
        constexpr int i = decltype(idx)::value, bm = i / NB, bn = i % NB;
        if constexpr (kEpi == static_cast<int>(Epilogue::kF32Workspace))  // (stored straight from the accumulators)
          store_acc4<kEpi>(p, acc[bm][bn], m0c + wm + bm * 16 + l16e, n0c + wn + bn * 16 + 4 * q4e, s_tab);
        else
          store_acc4<kEpi>(p, acc_read(acc[bm][bn]), m0c + wm + bm * 16 + l16e, n0c + wn + bn * 16 + 4 * q4e, s_tab);
        __builtin_amdgcn_sched_barrier(0);
      });
      ct += G;
      if (ct < tiles) begin_tile(ct, l16e, q4e);
      // The fragments read ahead for the next K step are read again here, so that none of them has to outlive the
      // epilogue: it needs their registers.
      {
        const uint16_t *sA = smem + cur * kSlotElems, *sB = sA + OpA::kElems;
#pragma unroll
        for (int b = 0; b < MB; ++b) fa[0][b] = OpA::frag(sA, wm + b * 16, 0, lane);
#pragma unroll
        for (int b = 0; b < NB; ++b) fb[0][b] = OpB::frag(sB, wn + b * 16, 0, lane);
      }
    }
  }
  wait_vmcnt<0>();  // surplus loads must have landed before the workgroup gives its LDS back
}

}  // namespace
}  // namespace osdp
