/*
 * CPU oracle for the operator-split linear layer of OSDP (arXiv 2209.13258).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against.  It shares no code with the GPU path and
 * the GPU path never calls it.  Only tests, the smoke check and the bench's
 * cpu_baseline leg may build, load or run it.
 *
 * What it computes (paper, Section 3.3 "Operator Splitting"): a huge MatMul
 * operator Y = X.W whose weight is kept sharded N ways (ZeRO/FSDP style,
 * Section 2.2) is cut into `k` slices that are re-gathered and processed one
 * after another, so that only one slice of gathered weight is live at a time
 * and the gathered-weight peak falls from size(MatMul) to
 * size(MatMul)/slice_granularity.  The slices here are COLUMN slices of W
 * (output features): Y is the concatenation of the slice products, dW is the
 * concatenation of the slice gradients and dX is the sum of the slice
 * partials.  The recombined result is, by definition, the unsplit product,
 * so this file holds two independent routes:
 *
 *   definition route : reassemble W from its shards, then the textbook
 *                      triple loops for Y, dX, dW (fp64, ascending index);
 *   split route      : for each slice, gather it into a fresh buffer,
 *                      compute the slice's Y / dW / dX-partial, free it,
 *                      recombine; tracks the peak number of live staging
 *                      bytes.
 *
 * The paper's own wording cuts the REDUCTION dimension instead (rows of W)
 * and sums the slice outputs; that variant is the second split route below
 * (osdp_oracle_*_rows).  Both recombine to the same unsplit operator.
 *
 * Readings of points the paper leaves open (all restated in the design notes):
 *   - shard layout : flat row-major index f = r*O + c, shard length
 *                    L = ceil(I*O/N), element lives in shard f / L at offset
 *                    f % L; the tail of the last shard is zero padding.
 *   - slice bounds : c0_j = floor(j*O/k), c1_j = floor((j+1)*O/k).
 *   - k = 0        : "granularity 0" of Section 4.3 means no splitting; it is
 *                    treated as k = 1.
 *   - W is [I x O] row-major, no bias.
 *   - inputs are bf16 bit patterns; every product and sum is fp64.
 *
 * Pins (tests/test_oracle_*.py): exact rational arithmetic on tiny shapes,
 * numpy's float64 matmul as the library special case, closed forms (identity,
 * ones, rank one), the flat-parameter chunking of a tensor library for the
 * shard map, the paper's worked size example (Section 3.3) and the memory
 * curve of the slice-granularity figure (Section 4.3) for the staging law.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_API __attribute__((visibility("default")))

/* ---- bf16 widening: a bf16 is the upper half of an IEEE binary32 -------- */
ORACLE_API double osdp_oracle_bf16_to_f64(uint16_t b) {
  uint32_t u = ((uint32_t)b) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

ORACLE_API int osdp_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ---- size arithmetic (Section 3.3: gathered weight of one MatMul) ------- */
ORACLE_API int64_t osdp_oracle_weight_bytes(int64_t I, int64_t O, int64_t elem_bytes) {
  return I * O * elem_bytes;
}

/* ---- slice bounds -------------------------------------------------------- */
static int64_t eff_k(int64_t k) { return k <= 0 ? 1 : k; }

ORACLE_API void osdp_oracle_slice_range(int64_t O, int64_t k, int64_t j, int64_t *c0, int64_t *c1) {
  k = eff_k(k);
  *c0 = (j * O) / k;
  *c1 = ((j + 1) * O) / k;
}

/* Peak gathered-weight bytes when `slots` slices are live at once
 * (Section 3.3: size(MatMul)/slice_granularity for one live slice). */
ORACLE_API int64_t osdp_oracle_peak_staging_bytes(int64_t I, int64_t O, int64_t k, int64_t slots,
                                                  int64_t elem_bytes) {
  int64_t wmax = 0;
  k = eff_k(k);
  if (slots > k) slots = k;
  for (int64_t j = 0; j < k; ++j) {
    int64_t c0, c1;
    osdp_oracle_slice_range(O, k, j, &c0, &c1);
    if (c1 - c0 > wmax) wmax = c1 - c0;
  }
  return slots * wmax * I * elem_bytes;
}

/* ---- shard-major address map -------------------------------------------- */
ORACLE_API int64_t osdp_oracle_shard_len(int64_t I, int64_t O, int64_t N) {
  return (I * O + N - 1) / N;
}

ORACLE_API void osdp_oracle_locate(int64_t I, int64_t O, int64_t N, int64_t r, int64_t c,
                                   int64_t *shard, int64_t *offset) {
  int64_t L = osdp_oracle_shard_len(I, O, N);
  int64_t f = r * O + c;
  *shard = f / L;
  *offset = f % L;
}

/* Reassemble the dense row-major W[I x O] from its N shards. */
ORACLE_API void osdp_oracle_assemble(int64_t I, int64_t O, int64_t N,
                                     const uint16_t *const *shards, uint16_t *W) {
  for (int64_t r = 0; r < I; ++r)
    for (int64_t c = 0; c < O; ++c) {
      int64_t s, off;
      osdp_oracle_locate(I, O, N, r, c, &s, &off);
      W[r * O + c] = shards[s][off];
    }
}

/* Cut a dense row-major W[I x O] into N shards of length L (tail zeroed). */
ORACLE_API void osdp_oracle_shard(int64_t I, int64_t O, int64_t N, const uint16_t *W,
                                  uint16_t *const *shards) {
  int64_t L = osdp_oracle_shard_len(I, O, N);
  for (int64_t s = 0; s < N; ++s) memset(shards[s], 0, (size_t)L * sizeof(uint16_t));
  for (int64_t r = 0; r < I; ++r)
    for (int64_t c = 0; c < O; ++c) {
      int64_t s, off;
      osdp_oracle_locate(I, O, N, r, c, &s, &off);
      shards[s][off] = W[r * O + c];
    }
}

/* Gather column slice j: Ws[r, c] = W[r, c0_j + c], dense row-major [I x w_j]. */
ORACLE_API void osdp_oracle_gather_slice(int64_t I, int64_t O, int64_t N, int64_t k, int64_t j,
                                         const uint16_t *const *shards, uint16_t *Ws) {
  int64_t c0, c1;
  osdp_oracle_slice_range(O, k, j, &c0, &c1);
  int64_t w = c1 - c0;
  for (int64_t r = 0; r < I; ++r)
    for (int64_t c = 0; c < w; ++c) {
      int64_t s, off;
      osdp_oracle_locate(I, O, N, r, c0 + c, &s, &off);
      Ws[r * w + c] = shards[s][off];
    }
}

/* ---- definition route: textbook loops, fp64, ascending index ------------ */

/* Y[t,o] = sum_i X[t,i] * W[i,o].  X is [T x I] with leading dimension ldx,
 * W is [I x O] with leading dimension ldw, Y is [T x O] dense fp64. */
ORACLE_API void osdp_oracle_matmul_fwd(int64_t T, int64_t I, int64_t O, const uint16_t *X,
                                       int64_t ldx, const uint16_t *W, int64_t ldw, double *Y) {
#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < T; ++t) {
    double *y = Y + t * O;
    for (int64_t o = 0; o < O; ++o) y[o] = 0.0;
    for (int64_t i = 0; i < I; ++i) {
      double x = osdp_oracle_bf16_to_f64(X[t * ldx + i]);
      const uint16_t *w = W + i * ldw;
      for (int64_t o = 0; o < O; ++o) y[o] += x * osdp_oracle_bf16_to_f64(w[o]);
    }
  }
}

/* dX[t,i] = sum_o dY[t,o] * W[i,o]. */
ORACLE_API void osdp_oracle_matmul_dx(int64_t T, int64_t I, int64_t O, const uint16_t *dY,
                                      int64_t lddy, const uint16_t *W, int64_t ldw, double *dX) {
#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < T; ++t) {
    for (int64_t i = 0; i < I; ++i) {
      double acc = 0.0;
      for (int64_t o = 0; o < O; ++o)
        acc += osdp_oracle_bf16_to_f64(dY[t * lddy + o]) * osdp_oracle_bf16_to_f64(W[i * ldw + o]);
      dX[t * I + i] = acc;
    }
  }
}

/* dW[i,o] = sum_t X[t,i] * dY[t,o]. */
ORACLE_API void osdp_oracle_matmul_dw(int64_t T, int64_t I, int64_t O, const uint16_t *X,
                                      int64_t ldx, const uint16_t *dY, int64_t lddy, double *dW) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < I; ++i) {
    double *g = dW + i * O;
    for (int64_t o = 0; o < O; ++o) g[o] = 0.0;
    for (int64_t t = 0; t < T; ++t) {
      double x = osdp_oracle_bf16_to_f64(X[t * ldx + i]);
      const uint16_t *d = dY + t * lddy;
      for (int64_t o = 0; o < O; ++o) g[o] += x * osdp_oracle_bf16_to_f64(d[o]);
    }
  }
}

/* Unsplit operator from shards: reassemble W, then the three definitions.
 * Any of Y, dX, dW may be NULL to skip it (dY may be NULL if both grads are).
 * dW is dense row-major [I x O] fp64. Returns 0, or -1 on allocation failure. */
ORACLE_API int osdp_oracle_linear(int64_t T, int64_t I, int64_t O, int64_t N, const uint16_t *X,
                                  const uint16_t *dY, const uint16_t *const *shards, double *Y,
                                  double *dX, double *dW) {
  uint16_t *W = (uint16_t *)malloc((size_t)I * O * sizeof(uint16_t));
  if (!W) return -1;
  osdp_oracle_assemble(I, O, N, shards, W);
  if (Y) osdp_oracle_matmul_fwd(T, I, O, X, I, W, O, Y);
  if (dX) osdp_oracle_matmul_dx(T, I, O, dY, O, W, O, dX);
  if (dW) osdp_oracle_matmul_dw(T, I, O, X, I, dY, O, dW);
  free(W);
  return 0;
}

/* ---- split route (Section 3.3: partition, sequential compute, combine) --- */

typedef struct {
  int64_t live, peak;
} staging_meter;

static uint16_t *staging_alloc(staging_meter *m, int64_t bytes) {
  uint16_t *p = (uint16_t *)malloc((size_t)bytes);
  if (p) {
    m->live += bytes;
    if (m->live > m->peak) m->peak = m->live;
  }
  return p;
}

static void staging_free(staging_meter *m, uint16_t *p, int64_t bytes) {
  free(p);
  m->live -= bytes;
}

/* Forward: for each slice j in ascending order gather Ws_j, compute
 * Y_j = X.Ws_j, release Ws_j; Y is the concatenation of the Y_j.
 * peak_staging (optional) receives the largest number of gathered-weight
 * bytes that were live at once. */
ORACLE_API int osdp_oracle_split_fwd(int64_t T, int64_t I, int64_t O, int64_t N, int64_t k,
                                     const uint16_t *X, const uint16_t *const *shards, double *Y,
                                     int64_t *peak_staging) {
  staging_meter m = {0, 0};
  k = eff_k(k);
  for (int64_t j = 0; j < k; ++j) {
    int64_t c0, c1;
    osdp_oracle_slice_range(O, k, j, &c0, &c1);
    int64_t w = c1 - c0;
    if (w == 0) continue;
    int64_t bytes = I * w * (int64_t)sizeof(uint16_t);
    uint16_t *Ws = staging_alloc(&m, bytes);
    double *Yj = (double *)malloc((size_t)T * w * sizeof(double));
    if (!Ws || !Yj) { free(Ws); free(Yj); return -1; }
    osdp_oracle_gather_slice(I, O, N, k, j, shards, Ws);
    osdp_oracle_matmul_fwd(T, I, w, X, I, Ws, w, Yj);
    for (int64_t t = 0; t < T; ++t)
      memcpy(Y + t * O + c0, Yj + t * w, (size_t)w * sizeof(double));
    free(Yj);
    staging_free(&m, Ws, bytes);
  }
  if (peak_staging) *peak_staging = m.peak;
  return 0;
}

/* Backward: for each slice j in ascending order gather Ws_j again (the
 * forward copy was released), compute dW_j = X^T.dY_j and the partial
 * dXpart_j = dY_j.Ws_j^T, release Ws_j.  dW_j is written to its place in the
 * shard-major gradient (dW_shards[s], fp64, same address map as W; padding is
 * left untouched); dX = sum_j dXpart_j in ascending j. */
ORACLE_API int osdp_oracle_split_bwd(int64_t T, int64_t I, int64_t O, int64_t N, int64_t k,
                                     const uint16_t *X, const uint16_t *dY,
                                     const uint16_t *const *shards, double *dX,
                                     double *const *dW_shards, int64_t *peak_staging) {
  staging_meter m = {0, 0};
  k = eff_k(k);
  for (int64_t e = 0; e < T * I; ++e) dX[e] = 0.0;
  for (int64_t j = 0; j < k; ++j) {
    int64_t c0, c1;
    osdp_oracle_slice_range(O, k, j, &c0, &c1);
    int64_t w = c1 - c0;
    if (w == 0) continue;
    int64_t bytes = I * w * (int64_t)sizeof(uint16_t);
    uint16_t *Ws = staging_alloc(&m, bytes);
    double *dWj = (double *)malloc((size_t)I * w * sizeof(double));
    double *part = (double *)malloc((size_t)T * I * sizeof(double));
    if (!Ws || !dWj || !part) { free(Ws); free(dWj); free(part); return -1; }
    osdp_oracle_gather_slice(I, O, N, k, j, shards, Ws);
    osdp_oracle_matmul_dw(T, I, w, X, I, dY + c0, O, dWj);
    osdp_oracle_matmul_dx(T, I, w, dY + c0, O, Ws, w, part);
    for (int64_t r = 0; r < I; ++r)
      for (int64_t c = 0; c < w; ++c) {
        int64_t s, off;
        osdp_oracle_locate(I, O, N, r, c0 + c, &s, &off);
        dW_shards[s][off] = dWj[r * w + c];
      }
    for (int64_t e = 0; e < T * I; ++e) dX[e] += part[e];
    free(part);
    free(dWj);
    staging_free(&m, Ws, bytes);
  }
  if (peak_staging) *peak_staging = m.peak;
  return 0;
}

/* ---- split route along the reduction dimension ---------------------------
 * Section 3.3 as printed: the last dimension of the input and the first
 * dimension of the operator are cut into slices, the slices are computed one
 * after another and the results are summed.  Slice j holds the rows
 * [r0_j, r1_j) of W, r0_j = floor(j*I/k):
 *     Y                = sum_j X[:, r0_j:r1_j] . W[r0_j:r1_j, :]      (sum)
 *     dX[:, r0_j:r1_j] = dY . W[r0_j:r1_j, :]^T                       (concatenate)
 *     dW[r0_j:r1_j, :] = X[:, r0_j:r1_j]^T . dY                       (concatenate)
 */
ORACLE_API void osdp_oracle_row_slice_range(int64_t I, int64_t k, int64_t j, int64_t *r0, int64_t *r1) {
  k = eff_k(k);
  *r0 = (j * I) / k;
  *r1 = ((j + 1) * I) / k;
}

/* Gather row slice j: Ws[r, c] = W[r0_j + r, c], dense row-major [w_j x O]. */
ORACLE_API void osdp_oracle_gather_row_slice(int64_t I, int64_t O, int64_t N, int64_t k, int64_t j,
                                             const uint16_t *const *shards, uint16_t *Ws) {
  int64_t r0, r1;
  osdp_oracle_row_slice_range(I, k, j, &r0, &r1);
  for (int64_t r = r0; r < r1; ++r)
    for (int64_t c = 0; c < O; ++c) {
      int64_t s, off;
      osdp_oracle_locate(I, O, N, r, c, &s, &off);
      Ws[(r - r0) * O + c] = shards[s][off];
    }
}

ORACLE_API int64_t osdp_oracle_peak_staging_bytes_rows(int64_t I, int64_t O, int64_t k, int64_t slots,
                                                       int64_t elem_bytes) {
  int64_t wmax = 0;
  k = eff_k(k);
  if (slots > k) slots = k;
  for (int64_t j = 0; j < k; ++j) {
    int64_t r0, r1;
    osdp_oracle_row_slice_range(I, k, j, &r0, &r1);
    if (r1 - r0 > wmax) wmax = r1 - r0;
  }
  return slots * wmax * O * elem_bytes;
}

ORACLE_API int osdp_oracle_split_fwd_rows(int64_t T, int64_t I, int64_t O, int64_t N, int64_t k,
                                          const uint16_t *X, const uint16_t *const *shards, double *Y,
                                          int64_t *peak_staging) {
  staging_meter m = {0, 0};
  k = eff_k(k);
  for (int64_t e = 0; e < T * O; ++e) Y[e] = 0.0;
  for (int64_t j = 0; j < k; ++j) {
    int64_t r0, r1;
    osdp_oracle_row_slice_range(I, k, j, &r0, &r1);
    int64_t w = r1 - r0;
    if (w == 0) continue;
    int64_t bytes = w * O * (int64_t)sizeof(uint16_t);
    uint16_t *Ws = staging_alloc(&m, bytes);
    double *part = (double *)malloc((size_t)T * O * sizeof(double));
    if (!Ws || !part) { free(Ws); free(part); return -1; }
    osdp_oracle_gather_row_slice(I, O, N, k, j, shards, Ws);
    osdp_oracle_matmul_fwd(T, w, O, X + r0, I, Ws, O, part); /* X[:, r0:r1] . Ws */
    for (int64_t e = 0; e < T * O; ++e) Y[e] += part[e];
    free(part);
    staging_free(&m, Ws, bytes);
  }
  if (peak_staging) *peak_staging = m.peak;
  return 0;
}

ORACLE_API int osdp_oracle_split_bwd_rows(int64_t T, int64_t I, int64_t O, int64_t N, int64_t k,
                                          const uint16_t *X, const uint16_t *dY,
                                          const uint16_t *const *shards, double *dX,
                                          double *const *dW_shards, int64_t *peak_staging) {
  staging_meter m = {0, 0};
  k = eff_k(k);
  for (int64_t j = 0; j < k; ++j) {
    int64_t r0, r1;
    osdp_oracle_row_slice_range(I, k, j, &r0, &r1);
    int64_t w = r1 - r0;
    if (w == 0) continue;
    int64_t bytes = w * O * (int64_t)sizeof(uint16_t);
    uint16_t *Ws = staging_alloc(&m, bytes);
    double *dXj = (double *)malloc((size_t)T * w * sizeof(double));
    double *dWj = (double *)malloc((size_t)w * O * sizeof(double));
    if (!Ws || !dXj || !dWj) { free(Ws); free(dXj); free(dWj); return -1; }
    osdp_oracle_gather_row_slice(I, O, N, k, j, shards, Ws);
    osdp_oracle_matmul_dx(T, w, O, dY, O, Ws, O, dXj);      /* dY . Ws^T            */
    osdp_oracle_matmul_dw(T, w, O, X + r0, I, dY, O, dWj);  /* X[:, r0:r1]^T . dY   */
    for (int64_t t = 0; t < T; ++t)
      memcpy(dX + t * I + r0, dXj + t * w, (size_t)w * sizeof(double));
    for (int64_t r = 0; r < w; ++r)
      for (int64_t c = 0; c < O; ++c) {
        int64_t s, off;
        osdp_oracle_locate(I, O, N, r0 + r, c, &s, &off);
        dW_shards[s][off] = dWj[r * O + c];
      }
    free(dWj);
    free(dXj);
    staging_free(&m, Ws, bytes);
  }
  if (peak_staging) *peak_staging = m.peak;
  return 0;
}

/* ---- slices treated one by one: DP or ZDP ---------------------------------
 * Section 3.3, last paragraph: once an operator is cut into slices, each slice
 * can be given its own mode.  A ZDP slice lives in the shards and is gathered
 * before every use (as above); a DP slice is replicated, so it is used where it
 * lies and nothing is staged for it, and its gradient is a full (unsharded)
 * array of the slice's shape.  Bit j of zdp_mask set: slice j is ZDP.
 * w_dp[j] (DP slices only) is the slice, row-major with leading dimension
 * ld_dp: [I x w_j] for column slices, [h_j x O] for row slices (rows != 0);
 * dw_dp[j] receives its gradient in the same shape (fp64).  Entries of ZDP
 * slices in w_dp / dw_dp are not looked at, nor are the shards' elements that
 * belong to DP slices; dW_shards is written for ZDP slices only. */
static void slice_range_along(int64_t I, int64_t O, int64_t k, int rows, int64_t j, int64_t *a0, int64_t *a1) {
  if (rows) osdp_oracle_row_slice_range(I, k, j, a0, a1);
  else osdp_oracle_slice_range(O, k, j, a0, a1);
}

ORACLE_API int osdp_oracle_split_fwd_mixed(int64_t T, int64_t I, int64_t O, int64_t N, int64_t k, int rows,
                                           uint64_t zdp_mask, const uint16_t *X,
                                           const uint16_t *const *shards, const uint16_t *const *w_dp,
                                           int64_t ld_dp, double *Y, int64_t *peak_staging) {
  staging_meter m = {0, 0};
  k = eff_k(k);
  if (rows)
    for (int64_t e = 0; e < T * O; ++e) Y[e] = 0.0;
  for (int64_t j = 0; j < k; ++j) {
    int64_t a0, a1;
    slice_range_along(I, O, k, rows, j, &a0, &a1);
    int64_t w = a1 - a0;
    if (w == 0) continue;
    int zdp = (int)((zdp_mask >> j) & 1u);
    int64_t bytes = (rows ? w * O : I * w) * (int64_t)sizeof(uint16_t);
    uint16_t *Ws = NULL;
    const uint16_t *Wj;   /* the slice's weights and their leading dimension */
    int64_t ldw;
    if (zdp) {
      Ws = staging_alloc(&m, bytes);
      if (!Ws) return -1;
      if (rows) osdp_oracle_gather_row_slice(I, O, N, k, j, shards, Ws);
      else osdp_oracle_gather_slice(I, O, N, k, j, shards, Ws);
      Wj = Ws;
      ldw = rows ? O : w;
    } else {
      Wj = w_dp[j];
      ldw = ld_dp;
    }
    if (rows) {
      double *part = (double *)malloc((size_t)T * O * sizeof(double));
      if (!part) { free(Ws); return -1; }
      osdp_oracle_matmul_fwd(T, w, O, X + a0, I, Wj, ldw, part);
      for (int64_t e = 0; e < T * O; ++e) Y[e] += part[e];
      free(part);
    } else {
      double *Yj = (double *)malloc((size_t)T * w * sizeof(double));
      if (!Yj) { free(Ws); return -1; }
      osdp_oracle_matmul_fwd(T, I, w, X, I, Wj, ldw, Yj);
      for (int64_t t = 0; t < T; ++t)
        memcpy(Y + t * O + a0, Yj + t * w, (size_t)w * sizeof(double));
      free(Yj);
    }
    if (zdp) staging_free(&m, Ws, bytes);
  }
  if (peak_staging) *peak_staging = m.peak;
  return 0;
}

ORACLE_API int osdp_oracle_split_bwd_mixed(int64_t T, int64_t I, int64_t O, int64_t N, int64_t k, int rows,
                                           uint64_t zdp_mask, const uint16_t *X, const uint16_t *dY,
                                           const uint16_t *const *shards, const uint16_t *const *w_dp,
                                           int64_t ld_dp, double *dX, double *const *dW_shards,
                                           double *const *dw_dp, int64_t *peak_staging) {
  staging_meter m = {0, 0};
  k = eff_k(k);
  if (!rows)
    for (int64_t e = 0; e < T * I; ++e) dX[e] = 0.0;
  for (int64_t j = 0; j < k; ++j) {
    int64_t a0, a1;
    slice_range_along(I, O, k, rows, j, &a0, &a1);
    int64_t w = a1 - a0;
    if (w == 0) continue;
    int zdp = (int)((zdp_mask >> j) & 1u);
    int64_t sr = rows ? w : I, sc = rows ? O : w;   /* the slice is sr x sc */
    int64_t bytes = sr * sc * (int64_t)sizeof(uint16_t);
    uint16_t *Ws = NULL;
    const uint16_t *Wj;
    int64_t ldw;
    if (zdp) {
      Ws = staging_alloc(&m, bytes);
      if (!Ws) return -1;
      if (rows) osdp_oracle_gather_row_slice(I, O, N, k, j, shards, Ws);
      else osdp_oracle_gather_slice(I, O, N, k, j, shards, Ws);
      Wj = Ws;
      ldw = sc;
    } else {
      Wj = w_dp[j];
      ldw = ld_dp;
    }
    double *dWj = (double *)malloc((size_t)sr * sc * sizeof(double));
    double *part = (double *)malloc((size_t)T * sr * sizeof(double));   /* dY-side product, T x (rows of the slice) */
    if (!dWj || !part) { free(Ws); free(dWj); free(part); return -1; }
    if (rows) {
      osdp_oracle_matmul_dw(T, w, O, X + a0, I, dY, O, dWj);   /* X[:, a0:a1]^T . dY */
      osdp_oracle_matmul_dx(T, w, O, dY, O, Wj, ldw, part);    /* dY . Wj^T  -> dX[:, a0:a1] */
      for (int64_t t = 0; t < T; ++t)
        memcpy(dX + t * I + a0, part + t * w, (size_t)w * sizeof(double));
    } else {
      osdp_oracle_matmul_dw(T, I, w, X, I, dY + a0, O, dWj);   /* X^T . dY[:, a0:a1] */
      osdp_oracle_matmul_dx(T, I, w, dY + a0, O, Wj, ldw, part);
      for (int64_t e = 0; e < T * I; ++e) dX[e] += part[e];
    }
    for (int64_t r = 0; r < sr; ++r)
      for (int64_t c = 0; c < sc; ++c) {
        if (zdp) {
          int64_t s, off;
          osdp_oracle_locate(I, O, N, rows ? a0 + r : r, rows ? c : a0 + c, &s, &off);
          dW_shards[s][off] = dWj[r * sc + c];
        } else {
          dw_dp[j][r * ld_dp + c] = dWj[r * sc + c];
        }
      }
    free(part);
    free(dWj);
    if (zdp) staging_free(&m, Ws, bytes);
  }
  if (peak_staging) *peak_staging = m.peak;
  return 0;
}

/* ---- single entries of the definition, for spot checks at full size ------ */

/* out[n] = Y[rows[n], cols[n]] from the sharded W (no reassembly). */
ORACLE_API void osdp_oracle_sample_y(int64_t T, int64_t I, int64_t O, int64_t N, const uint16_t *X,
                                     const uint16_t *const *shards, int64_t n,
                                     const int64_t *rows, const int64_t *cols, double *out) {
  (void)T;
#pragma omp parallel for schedule(static)
  for (int64_t q = 0; q < n; ++q) {
    int64_t t = rows[q], o = cols[q];
    double acc = 0.0;
    for (int64_t i = 0; i < I; ++i) {
      int64_t s, off;
      osdp_oracle_locate(I, O, N, i, o, &s, &off);
      acc += osdp_oracle_bf16_to_f64(X[t * I + i]) * osdp_oracle_bf16_to_f64(shards[s][off]);
    }
    out[q] = acc;
  }
}

/* out[n] = dX[rows[n], cols[n]]  (rows index tokens, cols index in-features). */
ORACLE_API void osdp_oracle_sample_dx(int64_t T, int64_t I, int64_t O, int64_t N,
                                      const uint16_t *dY, const uint16_t *const *shards, int64_t n,
                                      const int64_t *rows, const int64_t *cols, double *out) {
  (void)T;
#pragma omp parallel for schedule(static)
  for (int64_t q = 0; q < n; ++q) {
    int64_t t = rows[q], i = cols[q];
    double acc = 0.0;
    for (int64_t o = 0; o < O; ++o) {
      int64_t s, off;
      osdp_oracle_locate(I, O, N, i, o, &s, &off);
      acc += osdp_oracle_bf16_to_f64(dY[t * O + o]) * osdp_oracle_bf16_to_f64(shards[s][off]);
    }
    out[q] = acc;
  }
}

/* out[n] = dW[rows[n], cols[n]]  (rows index in-features, cols out-features). */
ORACLE_API void osdp_oracle_sample_dw(int64_t T, int64_t I, int64_t O, const uint16_t *X,
                                      const uint16_t *dY, int64_t n, const int64_t *rows,
                                      const int64_t *cols, double *out) {
#pragma omp parallel for schedule(static)
  for (int64_t q = 0; q < n; ++q) {
    int64_t i = rows[q], o = cols[q];
    double acc = 0.0;
    for (int64_t t = 0; t < T; ++t)
      acc += osdp_oracle_bf16_to_f64(X[t * I + i]) * osdp_oracle_bf16_to_f64(dY[t * O + o]);
    out[q] = acc;
  }
}
