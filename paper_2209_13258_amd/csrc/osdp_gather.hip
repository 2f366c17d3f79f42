// Shard -> slice gather (arXiv 2209.13258, Section 3.3: each slice of the
// sharded weight is re-gathered on its own before it is used).
//
// On one GPU the N shards are N device buffers, so the all-gather of a slice
// becomes a strided copy: row r of the slice is w contiguous elements that
// start at flat index r*O + c0 of the shard-major matrix (a row slice, the reduction-dimension
// split, is the same copy with c0 = 0, w = O and a row offset).  The kernel is a
// pure 16-byte-vector copy and is bound by HBM bandwidth: it reads I*w*2
// bytes and writes I*w*2 bytes.
#include <algorithm>

#include "osdp_internal.h"

namespace osdp {

namespace {

constexpr int kThreads = 256;

// One thread moves kUnroll vectors of 8 bf16 per grid-stride step (all loads issued before the stores).  Vector v of
// the dense destination [I x w] is row v / vecs_per_row, column chunk
// v % vecs_per_row.
template <bool kRowBlock, int kUnroll>
__global__ __launch_bounds__(kThreads) void gather_slice_kernel(
    ShardTable shards, ShardLayout lay, uint32_t r0, uint64_t c0, uint32_t vecs_per_row, uint64_t total_vecs,
    uint4 *__restrict__ dst) {
  __shared__ const uint16_t *s_tab[OSDP_MAX_SHARDS];
  if (threadIdx.x < OSDP_MAX_SHARDS)
    s_tab[threadIdx.x] = static_cast<const uint16_t *>(shards.p[threadIdx.x]);
  __syncthreads();

  const uint64_t step = static_cast<uint64_t>(gridDim.x) * (kThreads * kUnroll);
  for (uint64_t base = static_cast<uint64_t>(blockIdx.x) * (kThreads * kUnroll); base < total_vecs;
       base += step) {
    uint4 val[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint64_t v = base + u * kThreads + threadIdx.x;
      if (v < total_vecs) {
        // total_vecs < 2^32 is checked by the host, so 32-bit division is enough here
        const uint32_t v32 = static_cast<uint32_t>(v);
        const uint32_t rd = v32 / vecs_per_row;  // row of the destination
        const uint32_t cv = v32 - rd * vecs_per_row;
        const uint32_t r = r0 + rd;              // row of the full matrix
        uint32_t s;
        uint64_t off;
        if (kRowBlock) {
          s = r / static_cast<uint32_t>(lay.rows_per_shard);
          off = static_cast<uint64_t>(r - s * lay.rows_per_shard) * lay.O + c0 + cv * 8u;
        } else {
          const uint64_t f = static_cast<uint64_t>(r) * lay.O + c0 + cv * 8u;
          s = static_cast<uint32_t>(f / static_cast<uint64_t>(lay.L));
          off = f - static_cast<uint64_t>(s) * lay.L;
        }
        val[u] = load_global16(s_tab[s] + off);
      }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint64_t v = base + u * kThreads + threadIdx.x;
      if (v < total_vecs) store_global16(dst + v, val[u]);
    }
  }
}

__global__ __launch_bounds__(kThreads) void fill16_kernel(uint4 *__restrict__ dst, uint64_t vecs, uint32_t pattern2) {
  const uint4 v = {pattern2, pattern2, pattern2, pattern2};
  const uint64_t step = static_cast<uint64_t>(gridDim.x) * kThreads;
  for (uint64_t i = static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x; i < vecs; i += step) dst[i] = v;
}

}  // namespace

hipError_t launch_fill16(void *dst, size_t bytes, uint16_t pattern, hipStream_t stream) {
  if (bytes == 0) return hipSuccess;
  if (bytes % 16 || reinterpret_cast<uintptr_t>(dst) % 16) return hipErrorInvalidValue;
  const uint64_t vecs = bytes / 16;
  const uint64_t blocks = std::min<uint64_t>((vecs + kThreads - 1) / kThreads, 4096);
  const uint32_t p2 = static_cast<uint32_t>(pattern) | (static_cast<uint32_t>(pattern) << 16);
  hipLaunchKernelGGL(fill16_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0, stream,
                     static_cast<uint4 *>(dst), vecs, p2);
  return hipGetLastError();
}

template <bool kRowBlock, int kUnroll>
void launch_one(const ShardTable &shards, const ShardLayout &layout, int64_t r0, int64_t c0, uint64_t vecs_per_row, uint64_t total,
                unsigned max_blocks, void *staging, hipStream_t stream) {
  uint64_t blocks = (total + kThreads * kUnroll - 1) / (kThreads * kUnroll);
  if (blocks > max_blocks) blocks = max_blocks;
  hipLaunchKernelGGL((gather_slice_kernel<kRowBlock, kUnroll>), dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0, stream,
                     shards, layout, static_cast<uint32_t>(r0), static_cast<uint64_t>(c0), static_cast<uint32_t>(vecs_per_row), total,
                     static_cast<uint4 *>(staging));
}

hipError_t launch_gather(const ShardTable &shards, const ShardLayout &layout, int64_t r0, int64_t rows, int64_t c0,
                         int64_t w, void *staging, hipStream_t stream) {
  const uint64_t vecs_per_row = static_cast<uint64_t>(w) / 8;
  const uint64_t total = static_cast<uint64_t>(rows) * vecs_per_row;
  if (total == 0) return hipSuccess;
  if (total >> 32) return hipErrorInvalidValue;  // the kernel divides a 32-bit vector index
  // measured on MI355X: one vector per thread and grid-stride step is fastest up to 128 MiB slices (2 MiB in 6 us,
  // 12.5 MiB in 6.4 us, 50 and 128 MiB at 6.3 TB/s read + write, 80 % of the HBM peak); beyond that 4 vectors per
  // thread with all loads ahead of the stores do slightly better (512 MiB: 5.3 against 5.1 TB/s)
  const unsigned max_blocks = 8192;
  const bool rb = layout.rows_per_shard > 0;
  if (total * 16 <= (256ull << 20)) {
    if (rb) launch_one<true, 1>(shards, layout, r0, c0, vecs_per_row, total, max_blocks, staging, stream);
    else launch_one<false, 1>(shards, layout, r0, c0, vecs_per_row, total, max_blocks, staging, stream);
  } else {
    if (rb) launch_one<true, 4>(shards, layout, r0, c0, vecs_per_row, total, max_blocks, staging, stream);
    else launch_one<false, 4>(shards, layout, r0, c0, vecs_per_row, total, max_blocks, staging, stream);
  }
  return hipGetLastError();
}

}  // namespace osdp
