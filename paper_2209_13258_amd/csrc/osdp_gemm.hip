// Slice GEMMs of the operator-split linear layer (arXiv 2209.13258, Section 3.3):
//   forward   Y[:, slice]  = X . Ws          A K-contiguous, B N-contiguous
//   dW        dW[:, slice] = X^T . dY_slice  A M-contiguous, B N-contiguous
//   dX        dX (+)= dY_slice . Ws^T        A K-contiguous, B K-contiguous
// bf16 operands, fp32 accumulation on the gfx950 matrix cores
// (v_mfma_f32_32x32x16_bf16), bf16 round-to-nearest-even outputs.
//
// Every kernel in this file feeds each output element the same sequence of
// MFMA operations: K is walked in ascending blocks of 16, and inside a block
// logical k = 8*g + e sits in lane group g, element e of both operands.  Tile
// shape therefore never changes a result bit, which is what makes Y and dW of
// a split operator bit-identical to the unsplit ones.
#include "osdp_internal.h"

namespace osdp {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

struct GemmParams {
  int32_t M, N, K;
  const uint16_t *A;
  int64_t lda;
  const uint16_t *B;
  int64_t ldb;
  void *C;
  int64_t ldc;
  const float *acc_in;
  int64_t ld_acc;
  ShardLayout lay;
  int64_t c0;
  ShardTable shards;
};

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x0040u);  // NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return static_cast<uint32_t>(f32_to_bf16_rne(lo)) | (static_cast<uint32_t>(f32_to_bf16_rne(hi)) << 16);
}

// ---------------------------------------------------------------------------
// Generic kernel: 128 x 128 x 32 tile, 4 waves of 64 x 64, single LDS buffer,
// every access bounds-checked.  Handles any M, N and any K that is a multiple
// of 8 (the tail of the last K block is zero-filled, which adds exact zeros).
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
  }
  const int tiles_m = (p.M + GBM - 1) / GBM;
  const int tm = blockIdx.x % tiles_m, tn = blockIdx.x / tiles_m;
  const int m0 = tm * GBM, n0 = tn * GBN;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
  const int l32 = lane & 31, g = lane >> 5;

  f32x16 acc[2][2];
#pragma unroll
  for (int bm = 0; bm < 2; ++bm)
#pragma unroll
    for (int bn = 0; bn < 2; ++bn) {
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[bm][bn][i] = 0.f;
      if (kAccIn) {
        const int m = m0 + wm + bm * 32 + l32;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n = n0 + wn + bn * 32 + 8 * q + 4 * g;
          if (m < p.M && n < p.N) {
            const float4 c = *reinterpret_cast<const float4 *>(p.acc_in + static_cast<int64_t>(m) * p.ld_acc + n);
            acc[bm][bn][4 * q + 0] = c.x;
            acc[bm][bn][4 * q + 1] = c.y;
            acc[bm][bn][4 * q + 2] = c.z;
            acc[bm][bn][4 * q + 3] = c.w;
          }
        }
      }
    }

  for (int k0 = 0; k0 < p.K; k0 += GBK) {
    uint4 va[2], vb[2];
    generic_load<kAK>(p.A, p.lda, p.M, m0, k0, p.K, va);
    generic_load<kBK>(p.B, p.ldb, p.N, n0, k0, p.K, vb);
    __syncthreads();  // the previous block's LDS reads are done
    generic_store_lds<kAK>(As, va);
    generic_store_lds<kBK>(Bs, vb);
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < GBK / 16; ++kk) {
      bf16x8 a[2], b[2];
#pragma unroll
      for (int bm = 0; bm < 2; ++bm)
        a[bm] = *reinterpret_cast<const bf16x8 *>(&As[wm + bm * 32 + l32][kk * 16 + g * 8]);
#pragma unroll
      for (int bn = 0; bn < 2; ++bn)
        b[bn] = *reinterpret_cast<const bf16x8 *>(&Bs[wn + bn * 32 + l32][kk * 16 + g * 8]);
      // Operands are passed swapped (B tile as the MFMA's first operand) so that a lane ends
      // up with 4 consecutive output columns of one output row: acc[i] is
      // C[m = l32][n = 8*(i/4) + 4*g + i%4] of the 32 x 32 block.
#pragma unroll
      for (int bm = 0; bm < 2; ++bm)
#pragma unroll
        for (int bn = 0; bn < 2; ++bn)
          acc[bm][bn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[bn], a[bm], acc[bm][bn], 0, 0, 0);
    }
  }

#pragma unroll
  for (int bm = 0; bm < 2; ++bm)
#pragma unroll
    for (int bn = 0; bn < 2; ++bn) {
      const int m = m0 + wm + bm * 32 + l32;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n0 + wn + bn * 32 + 8 * q + 4 * g;
        if (m >= p.M || n >= p.N) continue;
        const float c0 = acc[bm][bn][4 * q], c1 = acc[bm][bn][4 * q + 1], c2 = acc[bm][bn][4 * q + 2],
                    c3 = acc[bm][bn][4 * q + 3];
        if (kEpi == static_cast<int>(Epilogue::kF32Workspace)) {
          float4 o = {c0, c1, c2, c3};
          *reinterpret_cast<float4 *>(static_cast<float *>(p.C) + static_cast<int64_t>(m) * p.ldc + n) = o;
        } else {
          uint2 o = {pack_bf16x2(c0, c1), pack_bf16x2(c2, c3)};
          uint16_t *dst;
          if (kEpi == static_cast<int>(Epilogue::kBf16RowMajor)) {
            dst = static_cast<uint16_t *>(p.C) + static_cast<int64_t>(m) * p.ldc + n;
          } else {
            int s;
            int64_t off;
            if (p.lay.rows_per_shard > 0) {
              s = m / p.lay.rows_per_shard;
              off = static_cast<int64_t>(m - s * p.lay.rows_per_shard) * p.lay.O + p.c0 + n;
            } else {
              const int64_t f = static_cast<int64_t>(m) * p.lay.O + p.c0 + n;
              s = static_cast<int>(f / p.lay.L);
              off = f - static_cast<int64_t>(s) * p.lay.L;
            }
            dst = s_tab[s] + off;
          }
          *reinterpret_cast<uint2 *>(dst) = o;
        }
      }
    }
}

template <bool kAK, bool kBK>
hipError_t dispatch_generic(const GemmProblem &q, const GemmParams &p, hipStream_t stream) {
  const int tiles = ((p.M + GBM - 1) / GBM) * ((p.N + GBN - 1) / GBN);
  dim3 grid(tiles), block(256);
  const bool acc = q.acc_in != nullptr;
#define OSDP_LAUNCH(EPI, ACC)                                                                          \
  hipLaunchKernelGGL((gemm_generic_kernel<kAK, kBK, static_cast<int>(EPI), ACC>), grid, block, 0, stream, p)
  switch (q.epilogue) {
    case Epilogue::kBf16RowMajor:
      if (acc) OSDP_LAUNCH(Epilogue::kBf16RowMajor, true); else OSDP_LAUNCH(Epilogue::kBf16RowMajor, false);
      break;
    case Epilogue::kBf16ShardMajor:
      if (acc) return hipErrorInvalidValue;
      OSDP_LAUNCH(Epilogue::kBf16ShardMajor, false);
      break;
    case Epilogue::kF32Workspace:
      if (acc) OSDP_LAUNCH(Epilogue::kF32Workspace, true); else OSDP_LAUNCH(Epilogue::kF32Workspace, false);
      break;
  }
#undef OSDP_LAUNCH
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm(const GemmProblem &q, hipStream_t stream) {
  if (q.M <= 0 || q.N <= 0 || q.K <= 0) return hipSuccess;
  GemmParams p;
  p.M = q.M; p.N = q.N; p.K = q.K;
  p.A = static_cast<const uint16_t *>(q.A); p.lda = q.lda;
  p.B = static_cast<const uint16_t *>(q.B); p.ldb = q.ldb;
  p.C = q.C; p.ldc = q.ldc;
  p.acc_in = q.acc_in; p.ld_acc = q.ld_acc;
  p.lay = q.layout; p.c0 = q.c0; p.shards = q.shards;
  if (q.a_kcontig && !q.b_kcontig) return dispatch_generic<true, false>(q, p, stream);
  if (!q.a_kcontig && !q.b_kcontig) return dispatch_generic<false, false>(q, p, stream);
  if (q.a_kcontig && q.b_kcontig) return dispatch_generic<true, true>(q, p, stream);
  return dispatch_generic<false, true>(q, p, stream);
}

}  // namespace osdp
