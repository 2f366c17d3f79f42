// Slice GEMMs of the operator-split linear layer (arXiv 2209.13258, Section 3.3):
//   forward   Y[:, slice]  = X . Ws          A K-contiguous, B N-contiguous
//   dW        dW[:, slice] = X^T . dY_slice  A M-contiguous, B N-contiguous
//   dX        dX (+)= dY_slice . Ws^T        A K-contiguous, B K-contiguous
// bf16 operands, fp32 accumulation on the gfx950 matrix cores
// (v_mfma_f32_16x16x32_bf16), bf16 round-to-nearest-even outputs.
//
// Every kernel in this file feeds each output element the same sequence of
// MFMA operations: K is walked in ascending blocks of 32, and inside a block
// logical k = 8*q + e sits in lane group q, element e of both operands.  Tile
// shape therefore never changes a result bit, which is what makes Y and dW of
// a split operator bit-identical to the unsplit ones.
#include "gemm_common.h"
#include "gemm_dma.h"
#include "gemm_w4.h"
#include "gemm_w4p.h"

namespace osdp {

namespace {

// ---------------------------------------------------------------------------
// Generic kernel: 128 x 128 x 32 tile, 4 waves of 64 x 64, single LDS buffer,
// every access bounds-checked.  Handles any M, N and any K that is a multiple
// of 8 (the tail of the last K block is zero-filled, which adds exact zeros);
// K = 0 is the empty sum: it stores zeros (or acc_in) and reads neither operand.
// ---------------------------------------------------------------------------
constexpr int GBM = 128, GBN = 128, GBK = 32, GLDK = GBK + 8;

template <bool kKContig>
__device__ __forceinline__ void generic_load(const uint16_t *__restrict__ src, int64_t ld, int rows_lim,
                                             int row0, int k0, int K, uint4 (&v)[2]) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int id = tid + p * 256;
    int gr, gk;
    if (kKContig) {
      gr = row0 + (id >> 2);
      gk = k0 + (id & 3) * 8;
    } else {
      gk = k0 + (id >> 4);
      gr = row0 + (id & 15) * 8;
    }
    uint4 z = {0u, 0u, 0u, 0u};
    if (gr < rows_lim && gk < K) {
      const int64_t off = kKContig ? static_cast<int64_t>(gr) * ld + gk : static_cast<int64_t>(gk) * ld + gr;
      z = *reinterpret_cast<const uint4 *>(src + off);
    }
    v[p] = z;
  }
}

template <bool kKContig>
__device__ __forceinline__ void generic_store_lds(uint16_t (*S)[GLDK], const uint4 (&v)[2]) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int id = tid + p * 256;
    if (kKContig) {
      *reinterpret_cast<uint4 *>(&S[id >> 2][(id & 3) * 8]) = v[p];
    } else {
      const int kr = id >> 4, r = (id & 15) * 8;
      const uint32_t w[4] = {v[p].x, v[p].y, v[p].z, v[p].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        S[r + 2 * e][kr] = static_cast<uint16_t>(w[e] & 0xffffu);
        S[r + 2 * e + 1][kr] = static_cast<uint16_t>(w[e] >> 16);
      }
    }
  }
}

template <bool kAK, bool kBK, int kEpi, bool kAccIn>
__global__ __launch_bounds__(256) void gemm_generic_kernel(GemmParams p) {
  __shared__ __attribute__((aligned(16))) uint16_t As[GBM][GLDK];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[GBN][GLDK];
  __shared__ uint16_t *s_tab[OSDP_MAX_SHARDS];

  const int tid = threadIdx.x;
  if (kEpi == static_cast<int>(Epilogue::kBf16ShardMajor)) {
    if (tid < OSDP_MAX_SHARDS) s_tab[tid] = static_cast<uint16_t *>(p.shards.p[tid]);
    __syncthreads();  // with K = 0 the loop below, and its barriers, do not run
  }
  const int tiles_m = (p.M + GBM - 1) / GBM;
  // a launch split along K: part s of the grid takes its range of k and stores plane s (the planes lie one below the other)
  const int tiles = tiles_m * ((p.N + GBN - 1) / GBN);
  const int part = p.k_parts > 1 ? blockIdx.x / tiles : 0;
  const int bid = blockIdx.x - part * tiles;
  const int k_len = p.k_parts > 1 ? p.K / p.k_parts : p.K;
  const int k_begin = part * k_len, k_end = k_begin + k_len;
  const int plane_row = part * p.M;
  const int tm = bid % tiles_m, tn = bid / tiles_m;
  const int m0 = tm * GBM, n0 = tn * GBN;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
  const int l16 = lane & 15, q = lane >> 4;

  // acc[bm][bn][i] is C[m0 + wm + 16*bm + l16][n0 + wn + 16*bn + 4*q + i]
  f32x4 acc[4][4];
#pragma unroll
  for (int bm = 0; bm < 4; ++bm)
#pragma unroll
    for (int bn = 0; bn < 4; ++bn) {
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[bm][bn][i] = 0.f;
      if (kAccIn) {
        const int m = m0 + wm + bm * 16 + l16, n = n0 + wn + bn * 16 + 4 * q;
        if (m < p.M && n < p.N) {
          const float4 c = *reinterpret_cast<const float4 *>(p.acc_in + static_cast<int64_t>(m) * p.ld_acc + n);
          acc[bm][bn][0] = c.x;
          acc[bm][bn][1] = c.y;
          acc[bm][bn][2] = c.z;
          acc[bm][bn][3] = c.w;
        }
      }
    }

  for (int k0 = k_begin; k0 < k_end; k0 += GBK) {
    uint4 va[2], vb[2];
    generic_load<kAK>(p.A, p.lda, p.M, m0, k0, k_end, va);
    generic_load<kBK>(p.B, p.ldb, p.N, n0, k0, k_end, vb);
    __syncthreads();  // the previous block's LDS reads are done
    generic_store_lds<kAK>(As, va);
    generic_store_lds<kBK>(Bs, vb);
    __syncthreads();
    // one K step of 32 per block: lane (l16, q) holds k = k0 + 8*q + 0..7 of its row / column
    bf16x8 a[4], b[4];
#pragma unroll
    for (int bm = 0; bm < 4; ++bm) a[bm] = *reinterpret_cast<const bf16x8 *>(&As[wm + bm * 16 + l16][q * 8]);
#pragma unroll
    for (int bn = 0; bn < 4; ++bn) b[bn] = *reinterpret_cast<const bf16x8 *>(&Bs[wn + bn * 16 + l16][q * 8]);
#pragma unroll
    for (int bm = 0; bm < 4; ++bm)
#pragma unroll
      for (int bn = 0; bn < 4; ++bn) acc[bm][bn] = mma_16x16x32(a[bm], b[bn], acc[bm][bn]);
  }

#pragma unroll
  for (int bm = 0; bm < 4; ++bm)
#pragma unroll
    for (int bn = 0; bn < 4; ++bn) {
      const int m = m0 + wm + bm * 16 + l16, n = n0 + wn + bn * 16 + 4 * q;
      if (m >= p.M || n >= p.N) continue;  // N is a multiple of 8 and n of 4: the 4 columns are in or out together
      store_acc4<kEpi>(p, acc[bm][bn], plane_row + m, n, s_tab);
    }
}

template <bool kAK, bool kBK, int kEpi, bool kAccIn>
hipError_t launch_generic(const GemmParams &p, hipStream_t stream) {
  const int tiles = ((p.M + GBM - 1) / GBM) * ((p.N + GBN - 1) / GBN);
  const int parts = p.k_parts > 1 ? p.k_parts : 1;
  hipLaunchKernelGGL((gemm_generic_kernel<kAK, kBK, kEpi, kAccIn>), dim3(tiles * parts), dim3(256), 0, stream, p);
  return hipGetLastError();
}

// The kernels use more dynamic LDS than the default limit; the attribute is set once per kernel and device.
constexpr int kMaxDevices = 16;

template <class Kernel>
hipError_t allow_lds(Kernel kernel, size_t lds, bool (&configured)[kMaxDevices]) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if (!configured[dev]) {  // a benign race sets the same attribute twice
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            static_cast<int>(lds));
    if (e != hipSuccess) return e;
    configured[dev] = true;
  }
  return hipSuccess;
}

template <int BM, int BN, int WM, int WN, int BK, int kStages, bool kAK, bool kBK, int kEpi, bool kAccIn>
hipError_t launch_dma(const GemmParams &p, hipStream_t stream) {
  constexpr int kWaves = (BM / WM) * (BN / WN);
  constexpr size_t lds = static_cast<size_t>(kStages) * (BM + BN) * BK * sizeof(uint16_t);
  static_assert(lds + OSDP_MAX_SHARDS * 8 <= 160 * 1024, "tile does not fit the 160 KB of LDS");
  auto kernel = gemm_dma_kernel<BM, BN, WM, WN, BK, kStages, kAK, kBK, kEpi, kAccIn>;
  static bool configured[kMaxDevices] = {};
  hipError_t e = allow_lds(kernel, lds, configured);
  if (e != hipSuccess) return e;
  const int tiles_m = p.M / BM, tiles_n = p.N / BN;
  const int parts = p.k_parts > 1 ? p.k_parts : 1;
  hipLaunchKernelGGL(kernel, dim3(tiles_m * tiles_n * parts), dim3(kWaves * 64), lds, stream, p, tiles_m, tiles_n);
  return hipGetLastError();
}

// The four-wave 256 x 256 kernel: two K blocks of 64 in LDS (128 KB).
template <bool kAK, bool kBK, int kEpi, bool kAccIn, bool kCopy>
hipError_t launch_w4(const GemmParams &p, hipStream_t stream) {
  constexpr size_t lds = 2 * (256 + 256) * 64 * sizeof(uint16_t);
  static_assert(lds + 2 * OSDP_MAX_SHARDS * 8 <= 160 * 1024, "tile does not fit the 160 KB of LDS");
  auto kernel = gemm_w4_kernel<kAK, kBK, kEpi, kAccIn, kCopy>;
  static bool configured[kMaxDevices] = {};
  hipError_t e = allow_lds(kernel, lds, configured);
  if (e != hipSuccess) return e;
  const int tiles_m = p.M / 256, tiles_n = p.N / 256;
  const int parts = p.k_parts > 1 ? p.k_parts : 1;
  hipLaunchKernelGGL(kernel, dim3(tiles_m * tiles_n * parts), dim3(256), lds, stream, p, tiles_m, tiles_n);
  return hipGetLastError();
}

// Adds up the fp32 planes of a launch that was split along K, plane 0 first, and stores the sum through the
// launch's own epilogue.  One thread per 4 consecutive columns.
template <int kEpi>
__global__ __launch_bounds__(256)
void combine_parts_kernel(GemmParams p, const float *parts, int n_parts) {
  uint16_t *const *s_tab = nullptr;
  if constexpr (kEpi == static_cast<int>(Epilogue::kBf16ShardMajor)) {
    __shared__ uint16_t *tab[OSDP_MAX_SHARDS];
    if (threadIdx.x < OSDP_MAX_SHARDS) tab[threadIdx.x] = static_cast<uint16_t *>(p.shards.p[threadIdx.x]);
    __syncthreads();
    s_tab = tab;
  }
  const int64_t plane = static_cast<int64_t>(p.M) * p.N;
  const int64_t v = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (v * 4 >= plane) return;
  const int per_row = p.N / 4;
  const int m = static_cast<int>(v / per_row), n = static_cast<int>(v - static_cast<int64_t>(m) * per_row) * 4;
  const float4 *src = reinterpret_cast<const float4 *>(parts) + v;
  float4 a = src[0];
  for (int s = 1; s < n_parts; ++s) {
    const float4 b = src[static_cast<int64_t>(s) * (plane / 4)];
    a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
  }
  const f32x4 c = {a.x, a.y, a.z, a.w};
  store_acc4<kEpi>(p, c, m, n, s_tab);
}

constexpr int kCUs = 256;

thread_local int64_t t_persistent_launches = 0;

// The persistent form of the four-wave kernel: one workgroup per CU walks through the tiles.
template <bool kAK, bool kBK, int kEpi, bool kAccIn>
hipError_t launch_w4p(const GemmParams &p, hipStream_t stream) {
  constexpr size_t lds = 2 * (256 + 256) * 64 * sizeof(uint16_t);
  auto kernel = gemm_w4p_kernel<kAK, kBK, kEpi, kAccIn>;
  static bool configured[kMaxDevices] = {};
  hipError_t e = allow_lds(kernel, lds, configured);
  if (e != hipSuccess) return e;
  const int tiles_m = p.M / 256, tiles_n = p.N / 256;
  const int tiles = tiles_m * tiles_n * (p.k_parts > 1 ? p.k_parts : 1);
  hipLaunchKernelGGL(kernel, dim3(tiles < kCUs ? tiles : kCUs), dim3(256), lds, stream, p, tiles_m, tiles_n);
  t_persistent_launches += 1;
  return hipGetLastError();
}

constexpr int kShortK = 1024;
constexpr int kW4MinK = 192;  // the four-wave kernel's K loop assumes at least three K blocks of 64
constexpr int kW4MinKdW = 8192;

// Estimated cost of covering M x N with BM x BN tiles on 256 CUs: tiles per CU times the tile's area, with a
// penalty for the lower MFMA efficiency of smaller tiles.  Tiles that run two to a CU were measured in pairs; a
// CU's odd last tile runs alone and slower, which is priced as one and a half tiles.  0 when the tile does not
// divide the problem.
double tile_cost(int M, int N, int BM, int BN, double penalty, int parts = 1) {
  if (M % BM || N % BN) return 0.0;
  const long tiles = static_cast<long>(M / BM) * (N / BN) * parts;
  const long per_cu = (tiles + kCUs - 1) / kCUs;
  const bool two_per_cu = BM * BN < 256 * 256;
  const double units = (two_per_cu && per_cu % 2) ? static_cast<double>(per_cu) + 0.5 : static_cast<double>(per_cu);
  return units * BM * BN * penalty;
}

bool fast_path(int M, int N, int K, int k_split, int n_split) {
  const bool generic = debug_options().gemm_generic.load(std::memory_order_relaxed) != 0;  // testing: the bounds-checked kernel
  return !generic && M % 128 == 0 && N % 128 == 0 && K > 0 && K % 64 == 0 && k_split % 64 == 0 &&
         n_split % 128 == 0;
}

// Tile shapes of the unchecked kernel and their measured cost per unit of tile area relative to 256 x 256, for
// the three operand layouts (forward, dW, dX).
struct TileShape {
  int bm, bn;
  double penalty[3];
};
// 8192^3 on MI355X, forward / dW / dX in PFLOP/s, eight-wave kernels: 256x256 1.22 / 1.23 / 1.26; 256x128 (two
// workgroups per CU) 1.04 / 0.90 / 1.09; 128x256 (two per CU) 1.19 / 1.02 / 1.06; 128x128 (two per CU) 1.03 / 1.05 /
// 1.03.  The 256x256 tile runs on the four-wave kernel (gemm_w4.h) whenever K >= 192: 1.43 / 1.30 / 1.45 on the
// same problem, which is what the penalties of the other shapes are relative to.
// K block and LDS stages of the eight-wave kernels per layout, also measured: forward (transposing reads of B) runs
// best with K blocks of 64 in two stages, dW and dX on the 256x256 tile and dW on the 128x128 tile with K blocks of
// 32 in four stages.
// The smaller tiles are sized for two workgroups per CU.  A launch with no more tiles than CUs has one, and is
// then bound by the latency of its loads (1024x4096x8192 for dW on 128x128 tiles: 41 GB/s per CU with 48 KB in
// flight); it takes the CU's whole LDS for K blocks of 64 in three or four stages, 96 KB in flight: dW 100 -> 88 us,
// the forward launch over two 256-column slices with K = 4096 64 -> 52 us.  The lone 128x128 workgroup also runs
// as 8 waves of 32x64 rather than 4 of 64x64, two per SIMD (another 3-10 %; without the deep pipeline it made no
// difference).
constexpr TileShape kTiles[4] = {{256, 256, {1.0, 1.0, 1.0}},
                                 {256, 128, {1.37, 1.40, 1.33}},
                                 {128, 256, {1.21, 1.23, 1.37}},
                                 {128, 128, {1.39, 1.20, 1.40}}};

constexpr int layout_kind(bool a_kcontig, bool b_kcontig) { return (a_kcontig && !b_kcontig) ? 0 : (!a_kcontig ? 1 : 2); }

// Cheapest tile for M x N; a column split must fall on a tile boundary.  -1: none divides the problem.
// parts > 1: the launch has that many workgroups per tile (parts of the reduction); the cost is in tile passes over
// the whole reduction all the same, so the caller divides it by parts.
int best_tile(int M, int N, int n_split, int kind, double *cost, int parts = 1) {
  int best = -1;
  double best_cost = 0.0;
  for (int i = 0; i < 4; ++i) {
    if (n_split % kTiles[i].bn) continue;
    const double c = tile_cost(M, N, kTiles[i].bm, kTiles[i].bn, kTiles[i].penalty[kind], parts);
    if (c > 0.0 && (best < 0 || c < best_cost)) {
      best = i;
      best_cost = c;
    }
  }
  if (cost) *cost = best_cost;
  return best;
}

// ---- concatenating launches split along K ----------------------------------------------------------------------
// A slice of a wide operator applied to few tokens (4096 x 1024 x 32768) has few output tiles and a long reduction:
// most CUs get no 256 x 256 tile, and the 128 x 128 tiles that would occupy them run at 70 % of the large tile's
// rate.  The forward product of such an operator over column slices (and likewise dX over row slices) is therefore
// defined as the sum of kPartK-long parts of the reduction: the parts run side by side as one launch (grid = parts x tiles), each into its own fp32 plane, and a
// second kernel adds the planes, plane 0 first, and rounds to bf16.  The number of parts depends on the token count
// and the reduction length alone - never on the slice width, the tile shape or the kernel - so Y keeps the same bits
// for every k, as the unsplit operator (k = 1) runs the same parts.
// Measured on 4096 tokens, 32768 -> 8192, whole steps with parts of 16384 / 8192 / 4096 against none, in TFLOP/s:
// k = 8 two slots 1130 / 1122 / 1068 against 1082; k = 16 978 / 1017 / 981 against 987; k = 4 1181 / 1170 / 1107
// against 1187; k = 8 one slot 975 / 1020 / 979 against 986; k = 8 half slices 926 / 920 / 884 against 826.
constexpr int kPartK = 8192;          // length of a part
constexpr int kPartMaxTokens = 4096;  // more tokens than this fill the CUs with any slice width that is worth staging
constexpr int kMaxParts = 8;

int forward_k_parts(int64_t M, int64_t K) {
  if (debug_options().split_k.load(std::memory_order_relaxed) == 0) return 1;  // testing: one part always
  if (M <= 0 || M > kPartMaxTokens || K < 2 * kPartK) return 1;
  const int parts = static_cast<int>(std::min<int64_t>(K / kPartK, kMaxParts));
  return K % (static_cast<int64_t>(parts) * 64) ? 1 : parts;
}

// Estimated duration of the combining kernel: the planes read, the result written.
double combine_estimate_us(int64_t M, int64_t N, int parts) {
  return (4.0 * parts + 2.0) * static_cast<double>(M) * static_cast<double>(N) / 3.0e6 + 8.0;
}

// *carry: the launch has a gather to carry (GemmParams::job is filled in); cleared by the launch that takes it.
template <bool kAK, bool kBK, int kEpi, bool kAccIn>
hipError_t launch_best(const GemmParams &p, hipStream_t stream, bool *carry) {
  constexpr int kind = layout_kind(kAK, kBK);
  const int parts = p.k_parts > 1 ? p.k_parts : 1;  // parts of the reduction run as further tiles of the same launch
  if (fast_path(p.M, p.N, p.K / parts, p.k_split, p.n_split)) {
    int best = best_tile(p.M, p.N, p.n_split, kind, nullptr, parts);
    const int forced = debug_options().tile.load(std::memory_order_relaxed);  // testing: tile 0..3 when it divides the problem
    const bool force = forced >= 0 && forced <= 3;
    if (force) {
      const TileShape &f = kTiles[forced];
      if (p.M % f.bm == 0 && p.N % f.bn == 0 && p.n_split % f.bn == 0) best = forced;
    }
    // A dX launch with a short reduction whose fp32 partial sum comes from or goes to memory is bound by that
    // traffic, and with only a round or two of large tiles every CU loads, computes and stores in step with the
    // others: two smaller workgroups per CU overlap one's loads and stores with the other's MFMAs (8192 x 4096 with
    // K = 256: 62 -> 54 us; with 8 rounds of large tiles, 4096 x 32768, the large tile stays 7 % ahead).
    if (kind == 2 && (kAccIn || kEpi == static_cast<int>(Epilogue::kF32Workspace)) && p.K <= kShortK && best == 0 &&
        static_cast<long>(p.M / 256) * (p.N / 256) <= 2 * kCUs && !force) {
      if (p.N % 256 == 0 && p.n_split % 256 == 0) best = 2;
      else if (p.n_split % 128 == 0) best = 1;
    }
    // A launch of at most one tile per CU cannot hide the latency of its loads behind a second workgroup: it gets
    // the whole LDS for a deeper pipeline instead (twice the bytes in flight).
    const bool deep = best > 0 && static_cast<long>(p.M / kTiles[best].bm) * (p.N / kTiles[best].bn) * parts <= kCUs &&
                      debug_options().deep.load(std::memory_order_relaxed) != 0;  // testing: 0 keeps the shallow pipelines
    const int fw = debug_options().four_wave.load(std::memory_order_relaxed);  // testing: 0 never, 1 whenever it can
    switch (best) {
      case 0:
        // (dW, both operands MN-contiguous: twice the fragment-read instructions and a serial epilogue per wave;
        // measured through the library, the four-wave kernel is 4-9 % ahead from K = 8192 and 3 % behind at K = 4096)
        if (p.K / parts >= kW4MinK && fw != 0 && (fw == 1 || p.K >= (kind == 1 ? kW4MinKdW : kW4MinK))) {
          // More tiles than CUs: the persistent form overlaps each tile's start-up with its predecessor's end
          // (3-12 % per launch).  It takes no gather along: *carry stays as it is and the caller launches the
          // gather by itself, which measured better on every workload than keeping the plain kernel for its sake.
          const int pst = debug_options().persistent.load(std::memory_order_relaxed);  // testing: 0 never, 1 for any number of tiles
          if (pst != 0 && !(parts > 1 && (p.k_split || kAccIn)) &&
              (pst == 1 || static_cast<long>(p.M / 256) * (p.N / 256) * parts > kCUs))
            return launch_w4p<kAK, kBK, kEpi, kAccIn>(p, stream);
          if constexpr (!(kAK && kBK)) {  // dX launches read every staged slice there is: they never carry a gather
            if (*carry) {
              *carry = false;
              return launch_w4<kAK, kBK, kEpi, kAccIn, true>(p, stream);
            }
          }
          return launch_w4<kAK, kBK, kEpi, kAccIn, false>(p, stream);
        }
        if (kind == 0) return launch_dma<256, 256, 64, 128, 64, 2, kAK, kBK, kEpi, kAccIn>(p, stream);
        return launch_dma<256, 256, 64, 128, 32, 4, kAK, kBK, kEpi, kAccIn>(p, stream);
      case 1:
        if (deep) return launch_dma<256, 128, 64, 64, 64, 3, kAK, kBK, kEpi, kAccIn>(p, stream);
        return launch_dma<256, 128, 64, 64, 32, 3, kAK, kBK, kEpi, kAccIn>(p, stream);
      case 2:
        if (deep) return launch_dma<128, 256, 64, 64, 64, 3, kAK, kBK, kEpi, kAccIn>(p, stream);
        return launch_dma<128, 256, 64, 64, 32, 3, kAK, kBK, kEpi, kAccIn>(p, stream);
      case 3:
        if (deep) return launch_dma<128, 128, 32, 64, 64, 4, kAK, kBK, kEpi, kAccIn>(p, stream);  // 8 waves of 32 x 64
        if (kind == 1) return launch_dma<128, 128, 64, 64, 32, 4, kAK, kBK, kEpi, kAccIn>(p, stream);
        return launch_dma<128, 128, 64, 64, 64, 2, kAK, kBK, kEpi, kAccIn>(p, stream);
    }
  }
  if (p.k_split || p.n_split) return hipErrorInvalidValue;  // the bounds-checked kernel takes one B segment only
  return launch_generic<kAK, kBK, kEpi, kAccIn>(p, stream);
}

// Columns [n0, n1) of a one-segment problem as a problem of its own.
template <bool kBK, int kEpi>
GemmParams column_range(const GemmParams &p, int n0, int n1) {
  GemmParams s = p;
  s.N = n1 - n0;
  s.B = kBK ? p.B + static_cast<int64_t>(n0) * p.ldb : p.B + n0;
  if (kEpi == static_cast<int>(Epilogue::kBf16ShardMajor)) s.c0 = p.c0 + n0;
  else if (kEpi == static_cast<int>(Epilogue::kF32Workspace)) s.C = static_cast<float *>(p.C) + n0;
  else s.C = static_cast<uint16_t *>(p.C) + n0;
  if (p.acc_in) s.acc_in = p.acc_in + n0;
  return s;
}

// Rows [m0, m1) likewise.
template <bool kAK, int kEpi>
GemmParams row_range(const GemmParams &p, int m0, int m1) {
  GemmParams s = p;
  s.M = m1 - m0;
  s.A = kAK ? p.A + static_cast<int64_t>(m0) * p.lda : p.A + m0;
  if (kEpi == static_cast<int>(Epilogue::kBf16ShardMajor)) s.r0 = p.r0 + m0;
  else if (kEpi == static_cast<int>(Epilogue::kF32Workspace)) s.C = static_cast<float *>(p.C) + static_cast<int64_t>(m0) * p.ldc;
  else s.C = static_cast<uint16_t *>(p.C) + static_cast<int64_t>(m0) * p.ldc;
  if (p.acc_in) s.acc_in = p.acc_in + static_cast<int64_t>(m0) * p.ld_acc;
  return s;
}

// A problem whose 256 x 256 tiles fill the CUs a whole number of times plus a little is run as two launches:
// the part that makes (nearly) whole rounds on the large tile, and the remainder on whatever tile suits it
// (usually a small one that spreads it over all CUs).  Tile shape never changes a result bit, so neither does this.
// Returns the modelled cost (tile-area units) of the best plan for a one-segment M x N x K problem of the given
// layout; axis = 1: columns [0, cut) and [cut, N) are launched separately; axis = 0: rows; axis = -1: one launch.
double plan_launches(int M, int N, int K, int kind, int *axis, int *cut) {
  double whole = 0.0;
  *axis = -1;
  *cut = 0;
  if (best_tile(M, N, 0, kind, &whole) < 0) return 0.0;
  // testing: split_launch = 0 keeps every problem in one launch, as does a forced tile shape
  if (debug_options().split_launch.load(std::memory_order_relaxed) == 0 ||
      debug_options().tile.load(std::memory_order_relaxed) >= 0 || M % 256 || N % 256)
    return whole;
  const int tm = M / 256, tn = N / 256;
  const double between = 1.0e7 / K;  // about 5 us from one launch to the next, in the cost's units of tile area
  double best = 0.95 * whole;        // only for a clear gain
  double rest = 0.0;
  // candidate cuts: for every number of rounds r, the most tile columns (rows) that r rounds of large tiles hold
  for (int r = 1; r <= 16; ++r) {
    const int cn = static_cast<int>(static_cast<long>(kCUs) * r / tm);
    if (cn <= 0) continue;
    if (cn >= tn) break;
    if (best_tile(M, N - cn * 256, 0, kind, &rest) < 0) continue;
    const double c = tile_cost(M, cn * 256, 256, 256, 1.0) + rest + between;
    if (c < best) { best = c; *axis = 1; *cut = cn * 256; }
  }
  for (int r = 1; r <= 16; ++r) {
    const int cm = static_cast<int>(static_cast<long>(kCUs) * r / tn);
    if (cm <= 0) continue;
    if (cm >= tm) break;
    if (best_tile(M - cm * 256, N, 0, kind, &rest) < 0) continue;
    const double c = tile_cost(cm * 256, N, 256, 256, 1.0) + rest + between;
    if (c < best) { best = c; *axis = 0; *cut = cm * 256; }
  }
  return *axis >= 0 ? best : whole;
}

template <bool kAK, bool kBK, int kEpi, bool kAccIn>
hipError_t launch_planned(const GemmParams &p, hipStream_t stream, bool *carry, float *planes, size_t planes_bytes) {
  // (forward launches of column slices, and the dX launches of row slices, which have the same shape of problem:
  // few tokens, a slice's worth of output columns, the whole uncut dimension as the reduction)
  if constexpr (kAK && !kAccIn && kEpi == static_cast<int>(Epilogue::kBf16RowMajor)) {
    // (a caller that passes no planes asks for the one-part product: the forward of row slices, whose launches
    // continue one accumulator chain instead)
    const int parts = (p.k_split || !planes) ? 1 : forward_k_parts(p.M, p.K);
    if (parts > 1) {
      if (planes_bytes < static_cast<size_t>(parts) * p.M * p.N * 4) return hipErrorInvalidValue;
      constexpr int kF32 = static_cast<int>(Epilogue::kF32Workspace);
      GemmParams s = p;
      s.k_parts = parts;
      s.C = planes;
      s.ldc = p.N;
      hipError_t e = launch_best<kAK, kBK, kF32, false>(s, stream, carry);
      if (e != hipSuccess) return e;
      const int64_t vecs = static_cast<int64_t>(p.M) * p.N / 4;
      hipLaunchKernelGGL((combine_parts_kernel<kEpi>), dim3(static_cast<unsigned>((vecs + 255) / 256)), dim3(256), 0, stream, p,
                         static_cast<const float *>(planes), parts);
      return hipGetLastError();
    }
  }
  if (!p.k_split && !p.n_split && fast_path(p.M, p.N, p.K, 0, 0)) {
    int axis, cut;
    plan_launches(p.M, p.N, p.K, layout_kind(kAK, kBK), &axis, &cut);
    if (axis == 1) {
      hipError_t e = launch_best<kAK, kBK, kEpi, kAccIn>(column_range<kBK, kEpi>(p, 0, cut), stream, carry);
      if (e != hipSuccess) return e;
      return launch_best<kAK, kBK, kEpi, kAccIn>(column_range<kBK, kEpi>(p, cut, p.N), stream, carry);
    }
    if (axis == 0) {
      hipError_t e = launch_best<kAK, kBK, kEpi, kAccIn>(row_range<kAK, kEpi>(p, 0, cut), stream, carry);
      if (e != hipSuccess) return e;
      return launch_best<kAK, kBK, kEpi, kAccIn>(row_range<kAK, kEpi>(p, cut, p.M), stream, carry);
    }
  }
  return launch_best<kAK, kBK, kEpi, kAccIn>(p, stream, carry);
}

}  // namespace

bool gemm_takes_two_segments(int64_t M, int64_t N, int64_t k_first, int64_t k_second) {
  return fast_path(static_cast<int>(M), static_cast<int>(N), static_cast<int>(k_first + k_second), static_cast<int>(k_first), 0) &&
         k_first > 0 && k_second > 0;
}

bool gemm_takes_two_column_segments(int64_t M, int64_t n_first, int64_t n_second, int64_t K) {
  return n_first > 0 && n_second > 0 &&
         fast_path(static_cast<int>(M), static_cast<int>(n_first + n_second), static_cast<int>(K), 0, static_cast<int>(n_first)) &&
         best_tile(static_cast<int>(M), static_cast<int>(n_first + n_second), static_cast<int>(n_first), 0, nullptr) >= 0;
}

double gemm_estimate_us(int64_t M, int64_t N, int64_t K, bool forward_parts) {
  // one CU sustains about 5e6 flop per microsecond (1.3 PFLOP/s over 256 CUs) on 256 x 256 tiles
  // (one launch on its best tile: pricing the whole-rounds + remainder pair here instead was measured and made the
  // forward launch grouping of config 3 slightly worse)
  double cost = 0.0;
  if (fast_path(static_cast<int>(M), static_cast<int>(N), static_cast<int>(K), 0, 0) &&
      best_tile(static_cast<int>(M), static_cast<int>(N), 0, 0, &cost) >= 0) {
    const int parts = forward_parts ? forward_k_parts(M, K) : 1;
    if (parts > 1) {
      best_tile(static_cast<int>(M), static_cast<int>(N), 0, 0, &cost, parts);
      return cost / parts * 2.0 * static_cast<double>(K) / 5.0e6 + combine_estimate_us(M, N, parts) + 6.0;
    }
    return cost * 2.0 * static_cast<double>(K) / 5.0e6 + 6.0;
  }
  const double tiles = static_cast<double>((M + GBM - 1) / GBM) * static_cast<double>((N + GBN - 1) / GBN);
  const double rounds = static_cast<double>(static_cast<long>((tiles + kCUs - 1) / kCUs));
  return rounds * GBM * GBN * 5.0 * 2.0 * static_cast<double>(K) / 5.0e6 + 6.0;  // the checked kernel is about 5x slower per tile
}

int64_t gemm_persistent_launches() { return t_persistent_launches; }

size_t gemm_forward_parts_bytes(int64_t M, int64_t N, int64_t K) {
  const int parts = forward_k_parts(M, K);
  return parts > 1 && N > 0 ? static_cast<size_t>(parts) * static_cast<size_t>(M) * static_cast<size_t>(N) * 4 : 0;
}

hipError_t check_device() {
  static std::atomic<int8_t> verdict[kMaxDevices] = {};  // 0: not looked at, 1: fits, -1: does not
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  int8_t v = verdict[dev].load(std::memory_order_relaxed);
  if (v == 0) {
    int cus = 0, xcds = 0;
    if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
    if ((e = hipDeviceGetAttribute(&xcds, hipDeviceAttributeNumberOfXccs, dev)) != hipSuccess) return e;
    v = (cus == kCUs && xcds == kXcds) ? 1 : -1;
    verdict[dev].store(v, std::memory_order_relaxed);
  }
  return v > 0 ? hipSuccess : hipErrorInvalidDevice;
}

namespace {
hipError_t dispatch_gemm(const GemmProblem &q, hipStream_t stream, bool *carry) {
  GemmParams p{};
  p.M = q.M; p.N = q.N; p.K = q.K;
  p.A = static_cast<const uint16_t *>(q.A); p.lda = q.lda;
  p.B = static_cast<const uint16_t *>(q.B); p.ldb = q.ldb;
  p.C = q.C; p.ldc = q.ldc;
  p.acc_in = q.acc_in; p.ld_acc = q.ld_acc;
  p.lay = q.layout; p.c0 = q.c0; p.r0 = q.r0; p.shards = q.shards;
  p.B2 = static_cast<const uint16_t *>(q.B2); p.ldb2 = q.ldb2;
  p.k_split = q.B2 ? q.k_split : 0; p.n_split = q.B2 ? q.n_split : 0;
  if (*carry) {
    const GatherRequest &g = *q.carry;
    const uint64_t total = static_cast<uint64_t>(g.rows) * (static_cast<uint64_t>(g.w) / 8);
    if (g.w % 8 || (total >> 32) || (reinterpret_cast<uintptr_t>(g.staging) & 15u)) return hipErrorInvalidValue;
    p.job.src = g.shards; p.job.lay = g.layout;
    p.job.r0 = static_cast<uint32_t>(g.r0); p.job.c0 = static_cast<uint64_t>(g.c0);
    p.job.vecs_per_row = static_cast<uint32_t>(g.w / 8); p.job.total_vecs = total;
    p.job.dst = static_cast<uint4 *>(g.staging);
  }
  if ((p.k_split || p.n_split) && !q.a_kcontig) return hipErrorInvalidValue;  // dW never takes a second segment
  if (p.k_split && p.n_split) return hipErrorInvalidValue;
  float *planes = static_cast<float *>(q.parts);
  const size_t planes_bytes = q.parts_bytes;
  constexpr int kRow = static_cast<int>(Epilogue::kBf16RowMajor), kShard = static_cast<int>(Epilogue::kBf16ShardMajor),
                kF32 = static_cast<int>(Epilogue::kF32Workspace);
  const bool acc = q.acc_in != nullptr;
  // The three GEMMs of the split linear layer, with the four accumulate forms for forward and dX, are the only combinations built.
  if (q.a_kcontig && !q.b_kcontig) {                                               // forward (accumulating when the reduction dimension is split)
    if (q.epilogue == Epilogue::kBf16RowMajor) return acc ? launch_planned<true, false, kRow, true>(p, stream, carry, planes, planes_bytes) : launch_planned<true, false, kRow, false>(p, stream, carry, planes, planes_bytes);
    if (q.epilogue == Epilogue::kF32Workspace) return acc ? launch_planned<true, false, kF32, true>(p, stream, carry, planes, planes_bytes) : launch_planned<true, false, kF32, false>(p, stream, carry, planes, planes_bytes);
  }
  if (!q.a_kcontig && !q.b_kcontig && !acc) {                                      // dW: into the shards, or (DP slice) a plain array
    if (q.epilogue == Epilogue::kBf16ShardMajor) return launch_planned<false, false, kShard, false>(p, stream, carry, planes, planes_bytes);
    if (q.epilogue == Epilogue::kBf16RowMajor) return launch_planned<false, false, kRow, false>(p, stream, carry, planes, planes_bytes);
  }
  if (q.a_kcontig && q.b_kcontig) {                                                // dX
    if (q.epilogue == Epilogue::kBf16RowMajor) return acc ? launch_planned<true, true, kRow, true>(p, stream, carry, planes, planes_bytes) : launch_planned<true, true, kRow, false>(p, stream, carry, planes, planes_bytes);
    if (q.epilogue == Epilogue::kF32Workspace) return acc ? launch_planned<true, true, kF32, true>(p, stream, carry, planes, planes_bytes) : launch_planned<true, true, kF32, false>(p, stream, carry, planes, planes_bytes);
  }
  return hipErrorInvalidValue;
}
}  // namespace

hipError_t launch_gemm(const GemmProblem &q, hipStream_t stream) {
  if (q.M < 0 || q.N < 0 || q.K < 0) return hipErrorInvalidValue;
  const GatherRequest *g = q.carry;
  const bool has_gather = g && g->rows > 0 && g->w > 0;
  if (has_gather && !q.carried) return hipErrorInvalidValue;  // the caller must learn whether the gather is still to do
  bool carry = has_gather;
  if (q.M > 0 && q.N > 0) {  // else nothing to write; K == 0 still writes the empty sum
    const hipError_t e = dispatch_gemm(q, stream, &carry);
    if (e != hipSuccess) return e;
  }
  if (q.carried) *q.carried = has_gather && !carry;
  return hipSuccess;
}

}  // namespace osdp
