// Internal declarations shared by the host API and the kernel launchers of libosdp.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "osdp.h"

namespace osdp {

// 16- and 8-byte accesses through pointers that are known to be device (global) memory but that the compiler sees as
// generic, e.g. shard pointers fetched from a table in LDS: without the address space it emits FLAT instructions,
// which check the address against the LDS and scratch apertures and count on both memory counters.
typedef unsigned int osdp_u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int osdp_u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 load_global16(const void *p) {
  const osdp_u32x4 v = *(const __attribute__((address_space(1))) osdp_u32x4 *)(p);
  return uint4{v[0], v[1], v[2], v[3]};
}
__device__ __forceinline__ void store_global16(void *p, uint4 v) {
  *(__attribute__((address_space(1))) osdp_u32x4 *)(p) = osdp_u32x4{v.x, v.y, v.z, v.w};
}
__device__ __forceinline__ void store_global8(void *p, uint2 v) {
  *(__attribute__((address_space(1))) osdp_u32x2 *)(p) = osdp_u32x2{v.x, v.y};
}

// Device pointers of the N shard buffers, passed to kernels by value.
struct ShardTable {
  void *p[OSDP_MAX_SHARDS];
};

// Where the shard-major matrix W / dW [I x O] lives: element (r, c) has flat
// index f = r*O + c and sits in shard f / L at offset f % L.  When N divides I
// (rows_per_shard > 0) shard s holds rows [s*rows_per_shard, (s+1)*rows_per_shard).
struct ShardLayout {
  int64_t O;               // row length of the full matrix
  int64_t L;               // elements per shard
  int32_t N;
  int32_t rows_per_shard;  // I / N when N divides I, else 0 (general flat map)
};

enum class Epilogue : int32_t {
  kBf16RowMajor = 0,   // C -> bf16, row-major with ldc
  kBf16ShardMajor = 1, // C -> bf16, scattered into the shard-major layout at column offset c0
  kF32Workspace = 2    // C -> fp32, row-major with ldc (the dX accumulator between slices)
};

// A slice gather: Ws[r, c] = W[r0 + r, c0 + c] for r < rows, c < w, into the dense row-major staging [rows x w].
struct GatherRequest {
  ShardTable shards;
  ShardLayout layout;
  int64_t r0, rows, c0, w;
  void *staging;
};

// One GEMM launch: C[M x N] (+)= A[M x K] . B[K x N], bf16 inputs, fp32 accumulate.
struct GemmProblem {
  int32_t M, N, K;
  const void *A;     // a_kcontig: A[m*lda + k], else A[k*lda + m]
  int64_t lda;
  bool a_kcontig;
  const void *B;     // b_kcontig: B[n*ldb + k], else B[k*ldb + n]
  int64_t ldb;
  bool b_kcontig;
  // Optional second segment of B (same layout as B, leading dimension ldb2), so that one launch runs
  // over two staged slices: k_split > 0: rows k >= k_split of the product come from B2 (k counted from
  // k_split); n_split > 0: columns n >= n_split come from B2 (n counted from n_split).  Not both.
  const void *B2;
  int64_t ldb2;
  int32_t k_split;
  int32_t n_split;
  void *C;           // row-major outputs; unused for kBf16ShardMajor
  int64_t ldc;
  const float *acc_in;  // fp32 [M x N] with ld_acc added to the product first, or nullptr
  int64_t ld_acc;
  Epilogue epilogue;
  ShardLayout layout;   // kBf16ShardMajor only
  ShardTable shards;    // kBf16ShardMajor only
  int64_t c0;           // kBf16ShardMajor only: column offset of C inside the full matrix
  int64_t r0;           // kBf16ShardMajor only: row offset of C inside the full matrix
  // Optional: a gather (into a staging slot this launch does not read) that the launch may take along.  The
  // four-wave kernel runs it inside the launch, between its MFMAs, and sets *carried; any other kernel
  // leaves *carried false and the gather to the caller.  carried must be given when carry is.
  const GatherRequest *carry;
  bool *carried;
  // Room for the fp32 planes of a forward launch split along K (gemm_forward_parts_bytes says how much the
  // product needs; with less the launch fails).  nullptr: the product is computed in one part whatever its shape.
  void *parts;
  size_t parts_bytes;
};

// Enqueue on `stream`.  Returns hipSuccess or the launch error.
hipError_t launch_gemm(const GemmProblem &p, hipStream_t stream);

// Whether launch_gemm accepts a two-segment B (B2 / k_split) for an M x N product whose K range is
// k_first columns from B followed by k_second columns from B2.
bool gemm_takes_two_segments(int64_t M, int64_t N, int64_t k_first, int64_t k_second);

// Whether launch_gemm accepts a two-segment N-contiguous B (B2 / n_split): N = n_first + n_second columns.
bool gemm_takes_two_column_segments(int64_t M, int64_t n_first, int64_t n_second, int64_t K);

// Rough duration in microseconds of one M x N x K GEMM launch (tile rounds over the CUs at the
// throughput measured for each tile shape); only used to choose between launch groupings.
// forward_parts: the product is a forward launch over column slices, which runs in parts of the reduction when few
// tokens meet a long reduction.
double gemm_estimate_us(int64_t M, int64_t N, int64_t K, bool forward_parts = false);

// Launches of the calling thread that ran as the persistent four-wave kernel so far (for the profile).
int64_t gemm_persistent_launches();

// Bytes of fp32 planes that launch_gemm needs in GemmProblem::parts for a forward product (A K-contiguous, B
// N-contiguous, bf16 row-major result, no accumulator) of M x N x K; 0: that product is not split along K.  The
// number of parts is a function of M and K alone.
size_t gemm_forward_parts_bytes(int64_t M, int64_t N, int64_t K);

// Ws[r, c] = W[r0 + r, c0 + c] for r < rows, c < w; Ws dense row-major [rows x w].
hipError_t launch_gather(const ShardTable &shards, const ShardLayout &layout, int64_t r0, int64_t rows, int64_t c0,
                         int64_t w, void *staging, hipStream_t stream);

// Fills `bytes` (a multiple of 16) at dst (16-byte aligned) with the 16-bit pattern: the debug mode that poisons
// released staging slots.  A kernel, not a memset node, so that a captured graph replays it correctly.
hipError_t launch_fill16(void *dst, size_t bytes, uint16_t pattern, hipStream_t stream);

// Test and debug switches (osdp_debug_option), process-wide.  Each is read with one relaxed atomic load where it
// applies; the environment is consulted once, when the library is loaded, for their initial values.
struct DebugOptions {
  std::atomic<int32_t> gemm_generic{0};    // 1: every GEMM runs on the bounds-checked kernel
  std::atomic<int32_t> tile{-1};           // 0..3: force that tile shape where it divides the problem
  std::atomic<int32_t> deep{-1};           // 0: launches of at most one tile per CU keep the shallow pipelines
  std::atomic<int32_t> split_launch{-1};   // 0: no whole-rounds + remainder launches
  std::atomic<int32_t> fwd_pair{-1};       // 0: the forward never pairs staged slices; 1: whenever the kernel can
  std::atomic<int32_t> fused_gather{-1};   // 0: gathers always run as launches of their own (second stream where given)
  std::atomic<int32_t> four_wave{-1};      // 0: 256 x 256 tiles run on the eight-wave kernel; 1: on the four-wave kernel wherever it can
  std::atomic<int32_t> persistent{-1};     // 0: launches of more 256 x 256 tiles than CUs keep the plain four-wave kernel instead of its persistent form; 1: the persistent form for any number of tiles
  std::atomic<int32_t> split_k{-1};        // 0: forward products are never split along K (changes the bits of those that are)
  std::atomic<int32_t> poison_staging{0};  // 1: staging slots hold NaN patterns whenever no gathered slice is live in them
};
DebugOptions &debug_options();

// The kernels' tile maps and cost estimates are written for the MI355X's 256 CUs in 8 XCDs; hipErrorInvalidDevice
// when the current device is something else.  Checked once per device.
hipError_t check_device();

// Stores the message as the calling thread's last error (osdp_last_error) and returns `status`.
osdp_status report_error(osdp_status status, const char *message);

}  // namespace osdp
