// Device-side pieces shared by the GEMM kernels of libosdp: parameter block, bf16 rounding,
// the workgroup -> tile map, accumulator load and the three epilogues.
#pragma once
#include "osdp_internal.h"

namespace osdp {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// One matrix-core step of every GEMM kernel here: a 16 x 16 block of C gains the product over 32 consecutive k.
// Lane l supplies 8 consecutive k (8 * (l / 16) ..) of row / column l % 16 of each operand.  The operands are
// passed swapped (the B fragment first), so that lane l ends up with C[m = l % 16][n = 4 * (l / 16) + 0..3]:
// runs of 4 consecutive output columns.  All kernels use this one instruction with k ascending, which is what
// makes their results bit-identical whatever the tile shape.
__device__ __forceinline__ f32x4 mma_16x16x32(bf16x8 a_rows, bf16x8 b_cols, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(b_cols, a_rows, c, 0, 0, 0);
}

// A slice gather that rides along with a GEMM launch (four-wave kernel only): the copy Ws[r, c] = W[r0 + r, c0 + c]
// of osdp_gather.hip, cut into one piece of 256 vectors per workgroup and K block and issued between the
// MFMAs (it saves the launch, not the memory time: the kernel is bound by the same memory pipe).  dst is the dense destination, total_vecs its size in 16-byte vectors (below 2^32).
struct GatherJob {
  ShardTable src;
  ShardLayout lay;
  uint32_t r0;
  uint32_t vecs_per_row;
  uint64_t c0;
  uint64_t total_vecs;
  uint4 *dst;
};

struct GemmParams {
  int32_t M, N, K;
  const uint16_t *A;
  int64_t lda;
  const uint16_t *B;
  int64_t ldb;
  const uint16_t *B2;  // second B segment: K-contiguous B, rows k >= k_split; N-contiguous B, columns n >= n_split
  int64_t ldb2;
  int32_t k_split;     // 0: none
  int32_t n_split;     // 0: none
  int32_t k_parts;     // > 1 (fp32 workspace epilogue with ldc = N, no second K segment): the grid is k_parts times the
                       // tiles, part s takes k in [s K / k_parts, (s + 1) K / k_parts) and writes plane s of C ([M x N] fp32 each)
  void *C;
  int64_t ldc;
  const float *acc_in;
  int64_t ld_acc;
  ShardLayout lay;
  int64_t c0;          // shard-major epilogue: column of the full matrix where C starts
  int64_t r0;          // shard-major epilogue: row of the full matrix where C starts
  ShardTable shards;
  GatherJob job;       // only read by kernels instantiated to carry one
};

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  const uint32_t u = __builtin_bit_cast(uint32_t, f);
  const uint32_t rounded = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;  // nearest even; carries into the exponent correctly
  const uint32_t quiet = (u >> 16) | 0x0040u;                        // NaN stays NaN
  return static_cast<uint16_t>((u & 0x7fffffffu) > 0x7f800000u ? quiet : rounded);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return static_cast<uint32_t>(f32_to_bf16_rne(lo)) | (static_cast<uint32_t>(f32_to_bf16_rne(hi)) << 16);
}


// Tile index of this workgroup.  Workgroups are dealt round-robin to the 8 XCDs, each with its
// own L2, so consecutive logical tile ids are first mapped onto one XCD; logical ids then walk
// the tile grid in column-major groups of kGroupM tile rows, which keeps the tiles that run
// together on an XCD inside a small patch of A row panels and B column panels (4 measured best of 2..16).
constexpr int kXcds = 8;
constexpr int kGroupM = 4;

// Logical id of this workgroup: the ids an XCD runs are consecutive.
__device__ __forceinline__ int logical_block() {
  const int nb = gridDim.x, bid = blockIdx.x;
  const int xcd = bid % kXcds, idx = bid / kXcds;
  const int base = nb / kXcds, rem = nb % kXcds;
  return xcd * base + (xcd < rem ? xcd : rem) + idx;
}

__device__ __forceinline__ void tile_of_pid(int pid, int tiles_m, int tiles_n, int *tm, int *tn) {
  const int per_group = kGroupM * tiles_n;
  const int group = pid / per_group, in_group = pid - group * per_group;
  const int first_m = group * kGroupM;
  const int gm = (tiles_m - first_m) < kGroupM ? (tiles_m - first_m) : kGroupM;
  *tm = first_m + in_group % gm;
  *tn = in_group / gm;
}

__device__ __forceinline__ void tile_of_block(int tiles_m, int tiles_n, int *tm, int *tn) {
  tile_of_pid(logical_block(), tiles_m, tiles_n, tm, tn);
}

// Accumulator layout of one wave: acc[bm][bn][i] is C[m][n] with
//   m = m_base + 16*bm + l16,  n = n_base + 16*bn + 4*q + i        (l16 = lane % 16, q = lane / 16).
// No bounds checks: the caller's tile is full.
template <int MB, int NB>
__device__ __forceinline__ void load_acc_tile(const GemmParams &p, f32x4 (&acc)[MB][NB], int m_base, int n_base,
                                              int l16, int q) {
#pragma unroll
  for (int bm = 0; bm < MB; ++bm)
#pragma unroll
    for (int bn = 0; bn < NB; ++bn) {
      const float *src = p.acc_in + static_cast<int64_t>(m_base + bm * 16 + l16) * p.ld_acc + n_base + bn * 16 + 4 * q;
      const float4 c = *reinterpret_cast<const float4 *>(src);
      acc[bm][bn][0] = c.x;
      acc[bm][bn][1] = c.y;
      acc[bm][bn][2] = c.z;
      acc[bm][bn][3] = c.w;
    }
}

// Stores 4 consecutive columns of row m starting at column n according to the epilogue.
template <int kEpi>
__device__ __forceinline__ void store_acc4(const GemmParams &p, f32x4 c, int m, int n, uint16_t *const *s_tab) {
  if (kEpi == static_cast<int>(Epilogue::kF32Workspace)) {
    float4 o = {c[0], c[1], c[2], c[3]};
    *reinterpret_cast<float4 *>(static_cast<float *>(p.C) + static_cast<int64_t>(m) * p.ldc + n) = o;
    return;
  }
  uint2 o = {pack_bf16x2(c[0], c[1]), pack_bf16x2(c[2], c[3])};
  uint16_t *dst;
  if (kEpi == static_cast<int>(Epilogue::kBf16RowMajor)) {
    dst = static_cast<uint16_t *>(p.C) + static_cast<int64_t>(m) * p.ldc + n;
  } else {
    int s;
    int64_t off;
    const int row = m + static_cast<int>(p.r0);
    if (p.lay.rows_per_shard > 0) {
      s = row / p.lay.rows_per_shard;
      off = static_cast<int64_t>(row - s * p.lay.rows_per_shard) * p.lay.O + p.c0 + n;
    } else {
      const int64_t f = static_cast<int64_t>(row) * p.lay.O + p.c0 + n;
      s = static_cast<int>(f / p.lay.L);
      off = f - static_cast<int64_t>(s) * p.lay.L;
    }
    dst = s_tab[s] + off;
  }
  store_global8(dst, o);
}

template <int MB, int NB, int kEpi>
__device__ __forceinline__ void store_acc_tile(const GemmParams &p, const f32x4 (&acc)[MB][NB], int m_base, int n_base,
                                               int l16, int q, uint16_t *const *s_tab) {
#pragma unroll
  for (int bm = 0; bm < MB; ++bm)
#pragma unroll
    for (int bn = 0; bn < NB; ++bn)
      store_acc4<kEpi>(p, acc[bm][bn], m_base + bm * 16 + l16, n_base + bn * 16 + 4 * q, s_tab);
}

}  // namespace
}  // namespace osdp
