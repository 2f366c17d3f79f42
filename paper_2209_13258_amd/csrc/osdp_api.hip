// Host side of libosdp: argument validation, slice planning, the two-stream
// gather/GEMM pipeline and the optional per-kernel timing.
//
// Pipeline (arXiv 2209.13258, Section 3.3: slices are processed one after
// another so that their memory is released serially, and the re-gathering is
// overlapped with computation): the gather of slice j+1 runs on the copy
// stream into the staging slot that the GEMM of slice j-1 has released, while
// the GEMM of slice j runs on the compute stream.
#include <algorithm>
#include <cctype>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>
#include <utility>
#include <vector>

#include "osdp_internal.h"

namespace {

using namespace osdp;

thread_local std::string t_last_error;

osdp_status fail(osdp_status st, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  t_last_error = buf;
  return st;
}

osdp_status fail_hip(hipError_t e, const char *what) {
  return fail(OSDP_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

#define OSDP_HIP(call)                                     \
  do {                                                     \
    hipError_t e_ = (call);                                \
    if (e_ != hipSuccess) return fail_hip(e_, #call);      \
  } while (0)

constexpr size_t kSlotAlign = 256;
constexpr uint16_t kPoison = 0x7FC0;  // bf16 quiet NaN
size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---- slice planning ---------------------------------------------------------
// A range [c0, c1) along the split dimension of W: columns (output features), or rows (input features, the
// reduction dimension of the forward product) when Resolved::rows is set.  Also used for ranges of sub-slice indices.
struct Slice {
  int64_t c0, c1;
};

struct Resolved {
  int64_t T, I, O;
  int32_t N, k;
  bool rows;                 // W is cut along its rows (the reduction dimension) instead of its columns
  int64_t D;                 // the dimension of W that is not cut: I for column slices, O for row slices
  int32_t mode;              // resolved osdp_staging_mode (never AUTO)
  int32_t slots;             // staging slots in the workspace
  std::vector<Slice> sub;    // the ranges processed one after another
  // slices in DP mode (zdp_mask bit clear) are read from, and their gradient written to, the caller's replica
  bool any_dp;
  std::vector<uint8_t> dp;      // per sub-slice: 1 = its slice is in DP mode (no gather, no staging)
  std::vector<int32_t> owner;   // per sub-slice: index j of its slice
  std::vector<int64_t> start;   // per sub-slice: where its slice starts along the split dimension
  ShardLayout layout;
  size_t slot_bytes;         // one staging slot, rounded up to kSlotAlign
  size_t peak_staging;       // gathered-weight bytes live at the peak (unrounded)
  size_t acc_bytes;          // fp32 accumulator T x D (more than one accumulating launch: dX for column slices, Y for row slices)
  size_t parts_bytes;        // fp32 planes of the widest concatenating launch (forward of column slices, dX of row slices) when the product is split along K (0: it is not)
  // launch plan; every entry is a range [c0, c1) of sub-slice indices
  std::vector<Slice> fwd;    // forward GEMM launches: one sub-slice, or two staged ones in one launch
  std::vector<Slice> group;  // backward: sub-slices staged together
  std::vector<Slice> pass;   // backward: dX launches
  std::vector<Slice> dw;     // backward: dW launches (dW needs no staged weights, so these may span groups)
};

// Caller-owned replicas of the slices in DP mode: w[j] / dw[j] point at slice j's weights / gradient, row-major
// with leading dimension ld ([I x w_j] for column slices, [h_j x O] for row slices).
struct Replicas {
  const void *const *w;
  void *const *dw;
  int64_t ld;
};

// Rough duration of one gather launch in microseconds: read + write of the slice at 5.5 TB/s plus the launch
// (measured alone between GEMMs: 32 MiB slices 17 us, 64 MiB 28 us, 128 MiB 44 us, 2 MiB 6 us).
double gather_estimate_us(int64_t elems) { return 4.0 * static_cast<double>(elems) / 5.5e6 + 6.0; }
// A gather that rides along inside a GEMM launch slows that launch by nearly what the gather takes alone (measured:
// 64 MiB slices add 25 us to a 190 us launch, 28 us as a launch of their own); what it saves is the launch and its gap.
constexpr double kCarriedShare = 0.9;

void slice_bounds(int64_t len, int64_t k, int64_t j, int64_t *c0, int64_t *c1) {
  *c0 = (j * len) / k;
  *c1 = ((j + 1) * len) / k;
}

osdp_status check_shape(const osdp_shape *s) {
  if (!s) return fail(OSDP_ERR_INVALID_ARG, "shape is NULL");
  if (s->T < 0 || s->I <= 0 || s->O <= 0)
    return fail(OSDP_ERR_INVALID_ARG, "I, O must be positive and T non-negative (got T %lld, I %lld, O %lld)",
                (long long)s->T, (long long)s->I, (long long)s->O);
  if (s->N < 1) return fail(OSDP_ERR_INVALID_ARG, "N must be >= 1 (got %d)", s->N);
  if (s->k < 0) return fail(OSDP_ERR_INVALID_ARG, "k must be >= 0 (got %d)", s->k);
  return OSDP_OK;
}

// Resolves k, the split dimension and the staging mode, checks what the kernels need and lists the sub-slices.
// `overlap_possible`: two distinct streams were given (or, for the size query, assumed).
//
// With column slices the forward launches write disjoint column ranges of Y and the dX launches add up; with
// row slices it is the other way round (Y adds up over the slices, dX is written range by range).  Both cases
// are planned as "concatenating" and "accumulating" launches over the sub-slices.
//
// `rep` (calls only, not the size query): where the DP slices lie.  DP sub-slices that follow one another in memory
// (the halves of one slice; neighbouring slices inside one full-layout replica) need no staging and so no
// separation: they are merged into one sub-slice, which only removes launches (the size query, which cannot
// know, answers for the unmerged plan and is never below what the merged one needs).
osdp_status resolve(const osdp_shape *shape, const osdp_plan *plan, int32_t op_index, bool overlap_possible,
                    bool is_bwd, Resolved *r, bool allow_dp = false, const Replicas *rep = nullptr) {
  osdp_status st = check_shape(shape);
  if (st != OSDP_OK) return st;
  int64_t k = shape->k;
  int32_t mode = OSDP_STAGING_AUTO;
  bool rows = false, per_pass = false;
  const uint64_t *mask = nullptr;
  if (plan) {
    if (plan->n_ops <= 0) return fail(OSDP_ERR_INVALID_ARG, "plan->n_ops must be positive");
    if (op_index < 0 || op_index >= plan->n_ops)
      return fail(OSDP_ERR_INVALID_ARG, "op_index %d outside the plan's %d operators", op_index, plan->n_ops);
    if (plan->k_per_op) k = plan->k_per_op[op_index];
    if (k < 0) return fail(OSDP_ERR_INVALID_ARG, "plan k must be >= 0 (got %lld)", (long long)k);
    mode = plan->staging_per_op ? plan->staging_per_op[op_index] : plan->staging;
    if (mode < OSDP_STAGING_AUTO || mode > OSDP_STAGING_HALF)
      return fail(OSDP_ERR_INVALID_ARG, "unknown staging mode %d", mode);
    if (plan->zdp_mask) mask = plan->zdp_mask + op_index;
    if (plan->split_dim_per_op) {
      const uint8_t d = plan->split_dim_per_op[op_index];
      if (d != OSDP_SPLIT_OUT_FEATURES && d != OSDP_SPLIT_IN_FEATURES && d != OSDP_SPLIT_LONGER && d != OSDP_SPLIT_PER_PASS)
        return fail(OSDP_ERR_INVALID_ARG, "unknown split dimension %d", static_cast<int>(d));
      // (per pass: columns in the forward pass, rows in the backward pass, so that Y, dX and dW all concatenate)
      rows = d == OSDP_SPLIT_IN_FEATURES || (d == OSDP_SPLIT_LONGER && shape->I > shape->O) || (d == OSDP_SPLIT_PER_PASS && is_bwd);
      per_pass = d == OSDP_SPLIT_PER_PASS;
    }
  }
  if (k == 0) k = 1;
  const int64_t T = shape->T, I = shape->I, O = shape->O;
  const int64_t len = rows ? I : O;  // length of the split dimension
  if (k > len) return fail(OSDP_ERR_INVALID_ARG, "k = %lld exceeds %s = %lld", (long long)k, rows ? "I" : "O", (long long)len);
  uint64_t zdp = ~0ull;  // bit j set: slice j is gathered
  if (mask) {
    const uint64_t want = k >= 64 ? ~0ull : ((1ull << k) - 1ull);
    if ((*mask & want) != want) {
      if (k > 64) return fail(OSDP_ERR_UNSUPPORTED, "a zdp_mask with cleared bits covers at most 64 slices (k = %lld)", (long long)k);
      if (!allow_dp)
        return fail(OSDP_ERR_UNSUPPORTED, "slices in DP mode (zdp_mask with cleared bits) need the replicas: use the _mixed entry points");
      if (per_pass)
        return fail(OSDP_ERR_UNSUPPORTED, "slices in DP mode need one split dimension for both passes (a replica is laid out slice by slice)");
      zdp = *mask & want;
    }
  }
  const int32_t N = shape->N;
  if (T >= (1ll << 31) || I >= (1ll << 31) || O >= (1ll << 31))
    return fail(OSDP_ERR_UNSUPPORTED, "T, I, O must be below 2^31");
  if (N > OSDP_MAX_SHARDS) return fail(OSDP_ERR_UNSUPPORTED, "N = %d exceeds %d shards", N, OSDP_MAX_SHARDS);
  if (I % 8 || O % 8) return fail(OSDP_ERR_UNSUPPORTED, "I and O must be multiples of 8 (got %lld, %lld)", (long long)I, (long long)O);
  const int64_t L = (I * O + N - 1) / N;
  if (L % 8) return fail(OSDP_ERR_UNSUPPORTED, "shard length %lld is not a multiple of 8", (long long)L);

  if (mode == OSDP_STAGING_AUTO) mode = (overlap_possible && k > 1) ? OSDP_STAGING_DOUBLE : OSDP_STAGING_SINGLE;
  if (k == 1 && mode == OSDP_STAGING_DOUBLE) mode = OSDP_STAGING_SINGLE;

  const int64_t D = rows ? O : I;
  r->T = T; r->I = I; r->O = O; r->N = N; r->k = static_cast<int32_t>(k); r->mode = mode;
  r->rows = rows; r->D = D;
  r->layout.O = O; r->layout.L = L; r->layout.N = N;
  r->layout.rows_per_shard = (I % N == 0) ? static_cast<int32_t>(I / N) : 0;
  r->sub.clear();
  r->dp.clear(); r->owner.clear(); r->start.clear();
  r->any_dp = false;
  int64_t wmax = 0;  // widest gathered sub-slice
  const char *what = rows ? "rows" : "columns";
  for (int64_t j = 0; j < k; ++j) {
    int64_t c0, c1;
    slice_bounds(len, k, j, &c0, &c1);
    if (c0 % 8 || c1 % 8)
      return fail(OSDP_ERR_UNSUPPORTED, "slice %lld = [%lld, %lld) is not aligned to 8 %s", (long long)j, (long long)c0, (long long)c1, what);
    const bool is_dp = j < 64 && !((zdp >> j) & 1ull);
    r->any_dp = r->any_dp || is_dp;
    const int parts = mode == OSDP_STAGING_HALF ? 2 : 1;
    if (parts == 2 && (c1 - c0) % 16)
      return fail(OSDP_ERR_UNSUPPORTED, "half-slice staging needs slice widths that are multiples of 16 (slice %lld has %lld)", (long long)j, (long long)(c1 - c0));
    for (int h = 0; h < parts; ++h) {
      const int64_t a = c0 + h * (c1 - c0) / 2, b = parts == 2 && h == 0 ? c0 + (c1 - c0) / 2 : c1;
      r->sub.push_back({a, b});
      r->dp.push_back(is_dp ? 1 : 0);
      r->owner.push_back(static_cast<int32_t>(j));
      r->start.push_back(c0);
      if (!is_dp) wmax = std::max(wmax, b - a);
    }
  }
  if (rep && r->any_dp && rep->w && (!is_bwd || rep->dw)) {
    size_t out = 0;
    for (size_t j = 0; j < r->sub.size(); ++j) {
      bool joins = false;
      if (out > 0 && r->dp[j] && r->dp[out - 1]) {
        const int32_t a = r->owner[out - 1], b = r->owner[j];
        if (a == b) {
          joins = true;
        } else {
          // slice b starts exactly where the merged run ends, in the weights and (backward) in the gradients
          const int64_t len = r->sub[out - 1].c1 - r->start[out - 1];
          const int64_t step = rows ? len * rep->ld : len;
          joins = static_cast<const uint16_t *>(rep->w[b]) == static_cast<const uint16_t *>(rep->w[a]) + step &&
                  (!is_bwd || static_cast<const uint16_t *>(rep->dw[b]) == static_cast<const uint16_t *>(rep->dw[a]) + step);
        }
      }
      if (joins) {
        r->sub[out - 1].c1 = r->sub[j].c1;
      } else {
        r->sub[out] = r->sub[j]; r->dp[out] = r->dp[j]; r->owner[out] = r->owner[j]; r->start[out] = r->start[j];
        ++out;
      }
    }
    r->sub.resize(out); r->dp.resize(out); r->owner.resize(out); r->start.resize(out);
  }
  r->slots = (mode == OSDP_STAGING_SINGLE) ? 1 : 2;
  int64_t n_gathered = 0;
  for (uint8_t d : r->dp) n_gathered += d ? 0 : 1;
  // the gather kernel counts 16-byte vectors in 32 bits, and one copy may fill both slots
  if (static_cast<uint64_t>(D) * static_cast<uint64_t>(wmax) / 8 >= (1ull << 31))
    return fail(OSDP_ERR_UNSUPPORTED, "slice of %lld x %lld elements is too large for the gather kernel", (long long)D, (long long)wmax);
  const size_t slice_bytes = static_cast<size_t>(D) * static_cast<size_t>(wmax) * 2;
  r->slot_bytes = round_up(slice_bytes, kSlotAlign);
  r->peak_staging = slice_bytes * static_cast<size_t>(std::min<int64_t>(r->slots, n_gathered));
  const int64_t n = static_cast<int64_t>(r->sub.size());
  auto width = [&](int64_t j) { return r->sub[j].c1 - r->sub[j].c0; };
  auto span = [&](int64_t a, int64_t b) { return r->sub[b - 1].c1 - r->sub[a].c0; };
  // one launch over sub-slices [a, b): concatenating (T x span x D) or accumulating (T x D x span)
  auto concat_us = [&](int64_t a, int64_t b) { return gemm_estimate_us(T, span(a, b), D, /*forward_parts=*/!rows); };
  auto accum_us = [&](int64_t a, int64_t b) { return gemm_estimate_us(T, D, span(a, b)); };
  // Two neighbouring gathered sub-slices can always share a launch: they are gathered by one copy into the two
  // slots taken as one buffer and read as one slice.  When one of them is a DP slice (read in place) the launch
  // needs a kernel that takes B in two segments.
  auto can_pair = [&](bool concat, int64_t j) {
    if (!r->dp[j] && !r->dp[j + 1]) return true;
    return concat ? gemm_takes_two_column_segments(T, width(j), width(j + 1), D)
                  : gemm_takes_two_segments(T, D, width(j), width(j + 1));
  };
  const bool fwd_concat = !rows, bwd_concat = rows;

  // Forward: with two slots, two staged slices may share one GEMM launch (column slices: twice the columns, so
  // fewer half-empty rounds of tiles; row slices: one trip of the fp32 partial sum through the workspace less)
  // at the price of exposing their gathers; taken when the estimate says it pays.
  r->fwd.clear();
  // (with half-slice staging a launch over both halves is the one-slot schedule: one copy of the whole slice, one
  // GEMM; the estimate decides here too, because on one GPU a gather that overlaps costs the GEMM beside it what
  // it saves, while half-width launches have half the output tiles)
  bool pair_fwd = r->slots == 2 && n >= 2;
  if (pair_fwd) {
    double t_single = 0.0, t_pair = 0.0, t_carried = 0.0;
    const double acc_trip_us = 8.0 * static_cast<double>(T) * static_cast<double>(D) / 3.0e6;  // fp32 out and back in
    for (int64_t j = 0; j + 1 < n; j += 2) {
      pair_fwd = pair_fwd && can_pair(fwd_concat, j);
      if (!pair_fwd) break;
      // two gathered neighbours are staged by one copy; a DP slice is read in place and costs no copy
      const double exposed = (!r->dp[j] && !r->dp[j + 1]) ? gather_estimate_us(D * (width(j) + width(j + 1)))
                             : (r->dp[j] ? 0.0 : gather_estimate_us(D * width(j))) +
                               (r->dp[j + 1] ? 0.0 : gather_estimate_us(D * width(j + 1)));
      for (int64_t q = j; q < j + 2; ++q)
        if (!r->dp[q]) t_carried += (q == 0 ? 1.0 : kCarriedShare) * gather_estimate_us(D * width(q));
      if (fwd_concat) {
        t_single += concat_us(j, j + 1) + concat_us(j + 1, j + 2);
        t_pair += concat_us(j, j + 2) + exposed;
      } else {
        t_single += accum_us(j, j + 1) + accum_us(j + 1, j + 2) + acc_trip_us;
        t_pair += accum_us(j, j + 2) + exposed;
      }
    }
    // One launch per slice takes the next slice's gather along, which costs the launch nearly the gather's own
    // time (measured on config 4's operators, forward alone: 8192 -> 32768 at k = 8 in pairs 1691 us, singly with
    // carried gathers 1777 us, singly on one slot 1704 us), so ties go to the pairs, which also copy in fewer, larger
    // pieces.  With gathers as launches of their own on a second stream (measured on configs 2 to 5 with both choices
    // forced) sharing a launch was never slower and up to 6 % faster than the estimate predicted (two streams cost
    // events, and a gather kernel beside the GEMMs only takes turns with their tiles), so there it only loses when
    // the estimate puts it clearly behind, as it does when the gathers dwarf the GEMMs (few tokens).
    if (debug_options().fused_gather.load(std::memory_order_relaxed) != 0)
      pair_fwd = pair_fwd && t_pair <= 1.03 * (t_single + t_carried);
    else
      pair_fwd = pair_fwd && t_pair < 1.10 * t_single;
    const int forced = debug_options().fwd_pair.load(std::memory_order_relaxed);  // testing: 0 never pairs, 1 pairs whenever the kernel can
    if (forced == 0) pair_fwd = false;
    if (forced == 1) {
      pair_fwd = true;
      for (int64_t j = 0; j + 1 < n; j += 2) pair_fwd = pair_fwd && can_pair(fwd_concat, j);
    }
  }
  for (int64_t j = 0; j < n;) {
    const int64_t step = (pair_fwd && j + 1 < n) ? 2 : 1;
    r->fwd.push_back({j, j + step});
    j += step;
  }

  // Backward processes the sub-slices in groups of `slots` (all staged at once): one dX launch per group
  // when the widths allow it, else one per sub-slice.
  r->group.clear();
  r->pass.clear();
  for (int64_t g0 = 0; g0 < n; g0 += r->slots) {
    const int64_t g1 = std::min<int64_t>(n, g0 + r->slots);
    r->group.push_back({g0, g1});
    const bool fuse = (g1 - g0 == 2) && can_pair(bwd_concat, g0);
    if (fuse) r->pass.push_back({g0, g1});
    else
      for (int64_t j = g0; j < g1; ++j) r->pass.push_back({j, j + 1});
  }
  // dW uses no gathered weight (column slices: dW[:, cols] = X^T . dY[:, cols]; row slices: dW[rows, :] =
  // X[:, rows]^T . dY), so its launches need not follow the staging groups: the ranges of `per` consecutive
  // sub-slices share a launch, `per` chosen by the estimate.
  int64_t per = r->slots;
  {
    double best = -1.0;
    for (int64_t cand = r->slots; ; cand *= 2) {
      if (cand > n) cand = n;
      double t = 0.0;
      for (int64_t a = 0; a < n; a += cand) {
        const int64_t w = span(a, std::min(n, a + cand));
        t += rows ? gemm_estimate_us(w, O, T) : gemm_estimate_us(I, w, T);
      }
      // the gathers of a staging group ride along with a dW launch that starts in the group: groups without
      // one run theirs as launches of their own
      if (debug_options().fused_gather.load(std::memory_order_relaxed) != 0)
        for (int64_t g0 = 0; g0 < n; g0 += r->slots)
          if (g0 % cand != 0) t += gather_estimate_us(D * span(g0, std::min<int64_t>(n, g0 + r->slots)));
      if (best < 0.0 || t < 0.97 * best) { best = t; per = cand; }
      if (cand == n) break;
    }
  }
  r->dw.clear();
  if (!r->any_dp) {
    for (int64_t a = 0; a < n; a += per) r->dw.push_back({a, std::min(n, a + per)});
  } else {
    // a launch stays within one destination: the sharded gradient (runs of gathered sub-slices, at most `per`)
    // or one DP slice's own gradient array (the sub-slices of that slice)
    for (int64_t a = 0; a < n;) {
      int64_t b = a + 1;
      if (r->dp[a]) {
        while (b < n && r->dp[b] && r->owner[b] == r->owner[a]) ++b;
      } else {
        while (b < n && !r->dp[b] && b - a < per) ++b;
      }
      r->dw.push_back({a, b});
      a = b;
    }
  }
  const size_t accumulating = is_bwd ? (bwd_concat ? 0 : r->pass.size()) : (fwd_concat ? 0 : r->fwd.size());
  r->acc_bytes = accumulating > 1 ? static_cast<size_t>(T) * static_cast<size_t>(D) * 4 : 0;
  // Forward products of few tokens with a long reduction run as parts of the reduction side by side, each into
  // an fp32 plane of the launch's shape (with DP slices the launches may be merged at call time, up to all columns).
  r->parts_bytes = 0;
  if (!is_bwd && fwd_concat) {
    int64_t widest = 0;
    for (const Slice &l : r->fwd) widest = std::max(widest, span(l.c0, l.c1));
    if (r->any_dp) widest = O;
    r->parts_bytes = gemm_forward_parts_bytes(T, widest, D);
  }
  if (is_bwd && bwd_concat) {  // dX of row slices: the same shape of problem
    int64_t widest = 0;
    for (const Slice &l : r->pass) widest = std::max(widest, span(l.c0, l.c1));
    if (r->any_dp) widest = I;
    r->parts_bytes = gemm_forward_parts_bytes(T, widest, D);
  }
  return OSDP_OK;
}

// Staging slots, the fp32 partial sum, the planes of concatenating launches split along K.
size_t workspace_total(const Resolved &r) { return r.slot_bytes * r.slots + r.acc_bytes + r.parts_bytes; }

osdp_status fill_table(const void *const *ptrs, int32_t N, const char *name, ShardTable *t) {
  if (!ptrs) return fail(OSDP_ERR_INVALID_ARG, "%s is NULL", name);
  std::memset(t, 0, sizeof *t);
  for (int32_t s = 0; s < N; ++s) {
    if (!ptrs[s]) return fail(OSDP_ERR_INVALID_ARG, "%s[%d] is NULL", name, s);
    if (!aligned16(ptrs[s])) return fail(OSDP_ERR_UNSUPPORTED, "%s[%d] is not 16-byte aligned", name, s);
    t->p[s] = const_cast<void *>(ptrs[s]);
  }
  return OSDP_OK;
}

osdp_status check_matrix(const void *p, int64_t ld, int64_t cols, const char *name) {
  if (!p) return fail(OSDP_ERR_INVALID_ARG, "%s is NULL", name);
  if (ld < cols) return fail(OSDP_ERR_INVALID_ARG, "leading dimension of %s (%lld) is below its row length %lld", name, (long long)ld, (long long)cols);
  if (ld % 8) return fail(OSDP_ERR_UNSUPPORTED, "leading dimension of %s (%lld) is not a multiple of 8", name, (long long)ld);
  if (!aligned16(p)) return fail(OSDP_ERR_UNSUPPORTED, "%s is not 16-byte aligned", name);
  return OSDP_OK;
}

osdp_status device_ok() {
  const hipError_t e = check_device();
  if (e == hipErrorInvalidDevice)
    return fail(OSDP_ERR_UNSUPPORTED, "the current device is not an MI355X (256 compute units in 8 XCDs), which the kernels are written for");
  if (e != hipSuccess) return fail_hip(e, "querying the device");
  return OSDP_OK;
}

osdp_status check_workspace(const Resolved &r, const void *ws, size_t bytes) {
  if (!ws) return fail(OSDP_ERR_INVALID_ARG, "workspace is NULL");
  if (reinterpret_cast<uintptr_t>(ws) % kSlotAlign) return fail(OSDP_ERR_UNSUPPORTED, "workspace is not 256-byte aligned");
  const size_t need = workspace_total(r);
  if (bytes < need) return fail(OSDP_ERR_WORKSPACE, "workspace holds %zu bytes, %zu needed", bytes, need);
  return OSDP_OK;
}

// ---- events -----------------------------------------------------------------
// A cyclic pool of untimed events for the cross-stream edges, one pool per host thread and device.  An event
// may be re-recorded once the waits on its earlier record have been enqueued, which always holds here: the
// calling thread issues every wait within two pipeline steps (at most six pool steps) of the record, and no
// other thread takes events from its pool.  When a thread ends its events go to a process-wide free list, from
// which new threads draw before creating any, so that threads which come and go do not pile events up; the
// events themselves live until the process ends (destroying them from a thread-exit or process-exit handler
// would race with the runtime's own teardown).
constexpr int kEventDevices = 16;

struct EventFreeList {
  std::mutex mu;
  std::vector<hipEvent_t> ev[kEventDevices];
};
EventFreeList &event_free_list() {
  static EventFreeList *list = new EventFreeList;  // never destroyed: thread-exit handlers may run late
  return *list;
}

class EventPool {
 public:
  ~EventPool() {
    EventFreeList &fl = event_free_list();
    std::lock_guard<std::mutex> lock(fl.mu);
    for (int d = 0; d < kEventDevices; ++d) fl.ev[d].insert(fl.ev[d].end(), dev_[d].ev.begin(), dev_[d].ev.end());
  }
  hipError_t get(hipEvent_t *out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kEventDevices) return hipErrorInvalidDevice;
    PerDevice &d = dev_[dev];
    if (d.ev.size() < kPool) {
      hipEvent_t ev = nullptr;
      {
        EventFreeList &fl = event_free_list();
        std::lock_guard<std::mutex> lock(fl.mu);
        if (!fl.ev[dev].empty()) {
          ev = fl.ev[dev].back();
          fl.ev[dev].pop_back();
        }
      }
      if (!ev) {
        e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
        if (e != hipSuccess) return e;
      }
      d.ev.push_back(ev);
      *out = ev;
      return hipSuccess;
    }
    *out = d.ev[d.next];
    d.next = (d.next + 1) % kPool;
    return hipSuccess;
  }

 private:
  static constexpr size_t kPool = 64;
  struct PerDevice {
    std::vector<hipEvent_t> ev;
    size_t next = 0;
  };
  PerDevice dev_[kEventDevices];
};

thread_local EventPool g_events;

// after: everything enqueued on `from` so far; makes `to` wait for it
hipError_t edge(hipStream_t from, hipStream_t to) {
  hipEvent_t ev;
  hipError_t e = g_events.get(&ev);
  if (e != hipSuccess) return e;
  e = hipEventRecord(ev, from);
  if (e != hipSuccess) return e;
  return hipStreamWaitEvent(to, ev, 0);
}

// ---- per-kernel timing --------------------------------------------------------
struct TimedLaunch {
  int kind;
  hipEvent_t start, stop;
  double flops, bytes;
};

struct Profile {
  bool active = false;
  size_t max_launches = 0;
  std::vector<TimedLaunch> launches;
  std::vector<hipEvent_t> spare;  // timed events kept for reuse
  int64_t carried_launches = 0;   // gathers that ran inside a GEMM launch
  int64_t persistent_launches = 0;  // GEMM launches that ran as the persistent kernel
  double carried_bytes = 0.0;
  // filled by osdp_profile_end for osdp_profile_overlap: [start, stop) of every timed launch in ms from the first event
  std::vector<std::pair<double, double>> gemm_iv, gather_iv;
};

// Total length of the union of intervals (sorts its argument).
double union_length(std::vector<std::pair<double, double>> &iv) {
  std::sort(iv.begin(), iv.end());
  double total = 0.0, end = -1.0e300;
  for (const auto &i : iv) {
    if (i.second <= end) continue;
    total += i.second - std::max(i.first, end);
    end = i.second;
  }
  return total;
}

thread_local Profile t_profile;

hipError_t timed_event(hipEvent_t *ev) {
  if (!t_profile.spare.empty()) {
    *ev = t_profile.spare.back();
    t_profile.spare.pop_back();
    return hipSuccess;
  }
  return hipEventCreate(ev);
}

template <class F>
hipError_t timed(int kind, double flops, double bytes, hipStream_t stream, F &&launch) {
  Profile &pf = t_profile;
  if (!pf.active || pf.launches.size() >= pf.max_launches) return launch();
  TimedLaunch t{kind, nullptr, nullptr, flops, bytes};
  hipError_t e = timed_event(&t.start);
  if (e != hipSuccess) return e;
  e = timed_event(&t.stop);
  if (e != hipSuccess) return e;
  e = hipEventRecord(t.start, stream);
  if (e != hipSuccess) return e;
  e = launch();
  if (e != hipSuccess) return e;
  e = hipEventRecord(t.stop, stream);
  if (e != hipSuccess) return e;
  pf.launches.push_back(t);
  return hipSuccess;
}

hipError_t do_gather(const Resolved &r, const ShardTable &tab, const Slice &s, void *slot, hipStream_t stream) {
  const int64_t w = s.c1 - s.c0;
  const double bytes = 2.0 * static_cast<double>(r.D) * static_cast<double>(w) * 2.0;
  return timed(OSDP_KERNEL_GATHER, 0.0, bytes, stream, [&] {
    return r.rows ? launch_gather(tab, r.layout, s.c0, w, 0, r.O, slot, stream)
                  : launch_gather(tab, r.layout, 0, r.I, s.c0, w, slot, stream);
  });
}

// The gather of sub-slice range s into `slot`, as a request a GEMM launch can take along.
GatherRequest gather_request(const Resolved &r, const ShardTable &tab, const Slice &s, void *slot) {
  GatherRequest g{};
  g.shards = tab;
  g.layout = r.layout;
  const int64_t w = s.c1 - s.c0;
  if (r.rows) { g.r0 = s.c0; g.rows = w; g.c0 = 0; g.w = r.O; }
  else { g.r0 = 0; g.rows = r.I; g.c0 = s.c0; g.w = w; }
  g.staging = slot;
  return g;
}

hipError_t gather_now(const GatherRequest &g, hipStream_t stream) {
  return timed(OSDP_KERNEL_GATHER, 0.0, 4.0 * static_cast<double>(g.rows) * static_cast<double>(g.w), stream, [&] {
    return launch_gather(g.shards, g.layout, g.r0, g.rows, g.c0, g.w, g.staging, stream);
  });
}

// One GEMM launch; a gather attached to it (g.carry) runs inside the launch when its kernel can take it along, else
// as a launch of its own right behind it.
hipError_t do_gemm(int kind, const GemmProblem &g, hipStream_t stream) {
  const double M = g.M, N = g.N, K = g.K;
  const double out_bytes = g.epilogue == Epilogue::kF32Workspace ? 4.0 : 2.0;
  const double bytes = 2.0 * M * K + 2.0 * K * N + out_bytes * M * N + (g.acc_in ? 4.0 * M * N : 0.0);
  bool carried = false;
  GemmProblem q = g;
  q.carried = &carried;
  const int64_t persistent_before = gemm_persistent_launches();
  hipError_t e = timed(kind, 2.0 * M * N * K, bytes, stream, [&] { return launch_gemm(q, stream); });
  Profile &pf = t_profile;
  if (pf.active) pf.persistent_launches += gemm_persistent_launches() - persistent_before;
  if (e != hipSuccess || !g.carry) return e;
  if (!carried) return gather_now(*g.carry, stream);
  if (pf.active) {
    pf.carried_launches += 1;
    pf.carried_bytes += 4.0 * static_cast<double>(g.carry->rows) * static_cast<double>(g.carry->w);
  }
  return hipSuccess;
}

// The GEMM that consumes the staged sub-slices [j0, j1): one in B0, or two in B0 and B1.
//   forward : act = X,  out = Y;   backward : act = dY, out = dX.
// A column slice is [I x w] row-major, a row slice [w x O] row-major (staged: dense); the forward product reads
// it as B[k][n] = Ws[k][n], the backward one as B[k][n] = Ws[n][k].
// Concatenating launches (forward with column slices, dX with row slices) write columns [c0, c0 + span) of out.
// Accumulating launches (dX with column slices, forward with row slices) add act[:, c0 : c0 + span] . B to the
// running fp32 sum: launch `idx` of `count` reads the sum from `acc` unless it is the first and writes it back
// unless it is the last, which rounds into out.
// A slice's weights as the GEMM reads them: a staging slot, or (DP mode) the slice's place in the caller's replica.
struct WeightView {
  const void *p;
  int64_t ld;
};

GemmProblem weight_gemm(const Resolved &r, bool is_fwd, int j0, int j1, WeightView B0, WeightView B1, const void *act,
                        int64_t ld_act, void *out, int64_t ld_out, float *acc, size_t idx, size_t count) {
  const Slice &s0 = r.sub[j0];
  const int64_t w0 = s0.c1 - s0.c0, span = r.sub[j1 - 1].c1 - s0.c0;
  const bool two = j1 - j0 == 2 && B1.p != nullptr;  // B1.p == nullptr: both sub-slices lie in B0 as one slice
  const bool concat = is_fwd != r.rows;
  GemmProblem g{};
  g.M = static_cast<int32_t>(r.T);
  g.a_kcontig = true;
  g.lda = ld_act;
  g.B = B0.p; g.ldb = B0.ld; g.b_kcontig = !is_fwd;
  if (two) { g.B2 = B1.p; g.ldb2 = B1.ld; }
  if (concat) {
    g.N = static_cast<int32_t>(span); g.K = static_cast<int32_t>(r.D);
    g.A = act;
    if (two) g.n_split = static_cast<int32_t>(w0);
    g.C = static_cast<uint16_t *>(out) + s0.c0; g.ldc = ld_out;
    g.epilogue = Epilogue::kBf16RowMajor;
  } else {
    g.N = static_cast<int32_t>(r.D); g.K = static_cast<int32_t>(span);
    g.A = static_cast<const uint16_t *>(act) + s0.c0;
    if (two) g.k_split = static_cast<int32_t>(w0);
    if (idx > 0) { g.acc_in = acc; g.ld_acc = r.D; }
    if (idx + 1 == count) {
      g.C = out; g.ldc = ld_out; g.epilogue = Epilogue::kBf16RowMajor;
    } else {
      g.C = acc; g.ldc = r.D; g.epilogue = Epilogue::kF32Workspace;
    }
  }
  return g;
}

// dW over the sub-slices [j0, j1), written into the shard-major gradient: column slices give
// dW[:, c0:c1] = X^T . dY[:, c0:c1], row slices dW[c0:c1, :] = X[:, c0:c1]^T . dY.
// element offset of sub-slice j inside its slice's replica
int64_t replica_offset(const Resolved &r, const Replicas &rep, int j) {
  const int64_t d = r.sub[j].c0 - r.start[j];
  return r.rows ? d * rep.ld : d;
}

// where the GEMM finds sub-slice j: its staging slot, or its place in the replica
WeightView weights_of(const Resolved &r, const Replicas &rep, int j, const void *slot) {
  if (r.dp[j]) return {static_cast<const uint16_t *>(rep.w[r.owner[j]]) + replica_offset(r, rep, j), rep.ld};
  return {slot, r.rows ? r.O : r.sub[j].c1 - r.sub[j].c0};
}

// Two neighbouring gathered sub-slices j, j+1 staged as one slice across both slots.
bool staged_jointly(const Resolved &r, int j0, int j1) { return j1 - j0 == 2 && !r.dp[j0] && !r.dp[j0 + 1]; }
Slice joint_range(const Resolved &r, int j0) { return {r.sub[j0].c0, r.sub[j0 + 1].c1}; }
WeightView joint_view(const Resolved &r, int j0, const void *slots) {
  return {slots, r.rows ? r.O : r.sub[j0 + 1].c1 - r.sub[j0].c0};
}

GemmProblem dw_gemm(const Resolved &r, int j0, int j1, const void *X, int64_t ldx, const void *dY, int64_t lddy,
                    const ShardTable &gtab, const Replicas &rep) {
  const int64_t c0 = r.sub[j0].c0, c1 = r.sub[j1 - 1].c1;
  GemmProblem g{};
  g.K = static_cast<int32_t>(r.T);
  g.lda = ldx; g.a_kcontig = false;
  g.ldb = lddy; g.b_kcontig = false;
  if (r.rows) {
    g.M = static_cast<int32_t>(c1 - c0); g.N = static_cast<int32_t>(r.O);
    g.A = static_cast<const uint16_t *>(X) + c0; g.B = dY;
    g.r0 = c0;
  } else {
    g.M = static_cast<int32_t>(r.I); g.N = static_cast<int32_t>(c1 - c0);
    g.A = X; g.B = static_cast<const uint16_t *>(dY) + c0;
    g.c0 = c0;
  }
  if (r.dp[j0]) {  // the gradient of a DP slice is a plain array of the slice's shape
    g.C = static_cast<uint16_t *>(rep.dw[r.owner[j0]]) + replica_offset(r, rep, j0);
    g.ldc = rep.ld;
    g.epilogue = Epilogue::kBf16RowMajor;
    g.c0 = g.r0 = 0;
  } else {
    g.epilogue = Epilogue::kBf16ShardMajor;
    g.layout = r.layout; g.shards = gtab;
  }
  return g;
}

osdp_status check_replicas(const Resolved &r, const Replicas &rep, bool need_dw) {
  if (!r.any_dp) return OSDP_OK;
  if (!rep.w) return fail(OSDP_ERR_INVALID_ARG, "w_dp is NULL but the plan has slices in DP mode");
  if (need_dw && !rep.dw) return fail(OSDP_ERR_INVALID_ARG, "dw_dp is NULL but the plan has slices in DP mode");
  if (rep.ld % 8) return fail(OSDP_ERR_UNSUPPORTED, "ld_dp (%lld) is not a multiple of 8", (long long)rep.ld);
  for (size_t j = 0; j < r.sub.size(); ++j) {
    if (!r.dp[j] || (j > 0 && r.owner[j] == r.owner[j - 1])) continue;
    int64_t cols = r.O;
    if (!r.rows) {
      cols = 0;
      for (size_t q = j; q < r.sub.size() && r.owner[q] == r.owner[j]; ++q) cols += r.sub[q].c1 - r.sub[q].c0;
    }
    if (rep.ld < cols)
      return fail(OSDP_ERR_INVALID_ARG, "ld_dp (%lld) is below the %lld columns of slice %d", (long long)rep.ld, (long long)cols, r.owner[j]);
    const void *w = rep.w[r.owner[j]];
    if (!w) return fail(OSDP_ERR_INVALID_ARG, "w_dp[%d] is NULL", r.owner[j]);
    if (!aligned16(w)) return fail(OSDP_ERR_UNSUPPORTED, "w_dp[%d] is not 16-byte aligned", r.owner[j]);
    if (need_dw) {
      const void *g = rep.dw[r.owner[j]];
      if (!g) return fail(OSDP_ERR_INVALID_ARG, "dw_dp[%d] is NULL", r.owner[j]);
      if (!aligned16(g)) return fail(OSDP_ERR_UNSUPPORTED, "dw_dp[%d] is not 16-byte aligned", r.owner[j]);
    }
  }
  return OSDP_OK;
}

}  // namespace

namespace osdp {
osdp_status report_error(osdp_status status, const char *message) {
  t_last_error = message;
  return status;
}

namespace {
struct DebugSwitch {
  const char *name;
  std::atomic<int32_t> DebugOptions::*field;
  int32_t lo, hi;  // accepted values; the default of the field stands for "not set"
};
const DebugSwitch kSwitches[] = {
    {"gemm_generic", &DebugOptions::gemm_generic, 0, 1}, {"tile", &DebugOptions::tile, -1, 3},
    {"deep", &DebugOptions::deep, -1, 1},                {"split_launch", &DebugOptions::split_launch, -1, 1},
    {"fwd_pair", &DebugOptions::fwd_pair, -1, 1},        {"poison_staging", &DebugOptions::poison_staging, 0, 1},
    {"persistent", &DebugOptions::persistent, -1, 1},    {"split_k", &DebugOptions::split_k, -1, 1},          {"four_wave", &DebugOptions::four_wave, -1, 1},      {"fused_gather", &DebugOptions::fused_gather, -1, 1},
};
}  // namespace

DebugOptions &debug_options() {
  // initial values: OSDP_DEBUG_<NAME IN CAPITALS>=<integer> in the environment, read once
  static DebugOptions *opt = [] {
    DebugOptions *o = new DebugOptions;
    for (const DebugSwitch &sw : kSwitches) {
      std::string var = "OSDP_DEBUG_";
      for (const char *c = sw.name; *c; ++c) var += static_cast<char>(std::toupper(static_cast<unsigned char>(*c)));
      if (const char *v = std::getenv(var.c_str())) {
        char *end = nullptr;
        const long val = std::strtol(v, &end, 10);
        if (end != v && *end == 0 && val >= sw.lo && val <= sw.hi) (o->*sw.field).store(static_cast<int32_t>(val));
      }
    }
    return o;
  }();
  return *opt;
}
}  // namespace osdp

// =============================================================================
extern "C" {

const char *osdp_version(void) { return "libosdp 0.1 (gfx950)"; }

const char *osdp_last_error(void) { return t_last_error.c_str(); }

const char *osdp_strerror(osdp_status status) {
  switch (status) {
    case OSDP_OK: return "ok";
    case OSDP_ERR_INVALID_ARG: return "invalid argument";
    case OSDP_ERR_UNSUPPORTED: return "unsupported shape, alignment or plan";
    case OSDP_ERR_WORKSPACE: return "workspace too small";
    case OSDP_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

static osdp_status slice_range_along(const osdp_shape *shape, bool rows, int32_t slice_j, int64_t *c0, int64_t *c1) {
  osdp_status st = check_shape(shape);
  if (st != OSDP_OK) return st;
  if (!c0 || !c1) return fail(OSDP_ERR_INVALID_ARG, "range output pointer is NULL");
  const int64_t k = shape->k == 0 ? 1 : shape->k;
  const int64_t len = rows ? shape->I : shape->O;
  if (k > len) return fail(OSDP_ERR_INVALID_ARG, "k = %lld exceeds %s = %lld", (long long)k, rows ? "I" : "O", (long long)len);
  if (slice_j < 0 || slice_j >= k) return fail(OSDP_ERR_INVALID_ARG, "slice %d outside [0, %lld)", slice_j, (long long)k);
  slice_bounds(len, k, slice_j, c0, c1);
  return OSDP_OK;
}

osdp_status osdp_slice_range(const osdp_shape *shape, int32_t slice_j, int64_t *c0, int64_t *c1) {
  return slice_range_along(shape, false, slice_j, c0, c1);
}

osdp_status osdp_row_slice_range(const osdp_shape *shape, int32_t slice_j, int64_t *r0, int64_t *r1) {
  return slice_range_along(shape, true, slice_j, r0, r1);
}

osdp_status osdp_split_linear_workspace_bytes(const osdp_shape *shape, const osdp_plan *plan, int32_t op_index,
                                              int32_t is_bwd, size_t *total, size_t *peak_weight_staging) {
  // With OSDP_STAGING_AUTO the call decides between one and two slots by the streams it is given:
  // the answer covers both (peak staging is that of the two-slot case).
  Resolved two, one;
  osdp_status st = resolve(shape, plan, op_index, /*overlap_possible=*/true, is_bwd != 0, &two, /*allow_dp=*/true);
  if (st != OSDP_OK) return st;
  st = resolve(shape, plan, op_index, /*overlap_possible=*/false, is_bwd != 0, &one, /*allow_dp=*/true);
  if (st != OSDP_OK) return st;
  if (total) *total = std::max(workspace_total(two), workspace_total(one));
  if (peak_weight_staging) *peak_weight_staging = two.peak_staging;
  return OSDP_OK;
}

static osdp_status gather_one(const osdp_shape *shape, uint8_t split_dim, int32_t slice_j, const void *const *w_shards,
                              void *staging, void *stream) {
  Resolved r;
  osdp_plan plan = {1, nullptr, nullptr, OSDP_STAGING_SINGLE, &split_dim};
  osdp_status st = resolve(shape, &plan, 0, false, false, &r);
  if (st != OSDP_OK) return st;
  if (slice_j < 0 || slice_j >= r.k) return fail(OSDP_ERR_INVALID_ARG, "slice %d outside [0, %d)", slice_j, r.k);
  ShardTable tab;
  st = fill_table(w_shards, r.N, "w_shards", &tab);
  if (st != OSDP_OK) return st;
  if (!staging) return fail(OSDP_ERR_INVALID_ARG, "staging is NULL");
  if (!aligned16(staging)) return fail(OSDP_ERR_UNSUPPORTED, "staging is not 16-byte aligned");
  OSDP_HIP(do_gather(r, tab, r.sub[slice_j], staging, static_cast<hipStream_t>(stream)));
  return OSDP_OK;
}

osdp_status osdp_split_linear_gather_slice(const osdp_shape *shape, int32_t slice_j, const void *const *w_shards,
                                           void *staging, void *stream) {
  return gather_one(shape, OSDP_SPLIT_OUT_FEATURES, slice_j, w_shards, staging, stream);
}

osdp_status osdp_split_linear_gather_row_slice(const osdp_shape *shape, int32_t slice_j, const void *const *w_shards,
                                               void *staging, void *stream) {
  return gather_one(shape, OSDP_SPLIT_IN_FEATURES, slice_j, w_shards, staging, stream);
}

static osdp_status forward(const osdp_shape *shape, const osdp_plan *plan, int32_t op_index, bool allow_dp, const void *X,
                           int64_t ldx, const void *const *w_shards, const Replicas &rep, void *Y, int64_t ldy,
                           void *workspace, size_t workspace_bytes, void *stream_compute, void *stream_copy) {
  hipStream_t sc = static_cast<hipStream_t>(stream_compute), sp = static_cast<hipStream_t>(stream_copy);
  const bool two_streams = sp != nullptr && sp != sc;
  Resolved r;
  osdp_status st = resolve(shape, plan, op_index, two_streams, false, &r, allow_dp, &rep);
  if (st != OSDP_OK) return st;
  const bool no_tokens = r.T == 0;  // X and Y have no rows and may be NULL
  if (!no_tokens && (st = check_matrix(X, ldx, r.I, "X")) != OSDP_OK) return st;
  if (!no_tokens && (st = check_matrix(Y, ldy, r.O, "Y")) != OSDP_OK) return st;
  ShardTable tab;
  if ((st = fill_table(w_shards, r.N, "w_shards", &tab)) != OSDP_OK) return st;
  if ((st = check_replicas(r, rep, false)) != OSDP_OK) return st;
  if ((st = check_workspace(r, workspace, workspace_bytes)) != OSDP_OK) return st;
  if ((st = device_ok()) != OSDP_OK) return st;
  if (no_tokens) return OSDP_OK;  // Y is empty: nothing is gathered, nothing is launched

  char *ws = static_cast<char *>(workspace);
  float *acc = reinterpret_cast<float *>(ws + r.slot_bytes * r.slots);  // row slices: Y's fp32 partial sum
  void *planes = r.parts_bytes ? ws + r.slot_bytes * r.slots + r.acc_bytes : nullptr;  // planes of launches split along K
  const size_t planes_bytes = r.parts_bytes;
  const int n = static_cast<int>(r.sub.size());
  // Debug mode: a slot holds NaN patterns whenever no gathered slice is live in it, so that a GEMM that ran ahead
  // of its gather, or a gather that overwrote a slice still being read, shows up as NaN (or wrong) outputs.
  const bool poison = debug_options().poison_staging.load(std::memory_order_relaxed) != 0;
  if (poison) OSDP_HIP(launch_fill16(ws, r.slot_bytes * r.slots, kPoison, sc));
  // A launch over two staged sub-slices holds both slots, so the next gather has to wait for it whatever stream it
  // is on: with such launches there is nothing to overlap, and everything goes on the compute stream, event-free.
  bool pairs = false;
  for (const Slice &l : r.fwd) pairs = pairs || l.c1 - l.c0 == 2;
  // One launch per sub-slice and two slots: the GEMM of sub-slice j takes the gather of sub-slice j+1 along, into
  // the slot that the GEMM of sub-slice j-1 has finished with (it ran earlier on the same stream).  Only the first
  // gather is a launch of its own; nothing else is exposed, and no second stream or event is involved.
  const bool fused = r.slots == 2 && n > 1 && !pairs && debug_options().fused_gather.load(std::memory_order_relaxed) != 0;
  if (fused) {
    for (int j = 0; j < n; ++j) {
      void *slot = ws + static_cast<size_t>(j % 2) * r.slot_bytes;
      if (j == 0 && !r.dp[0]) OSDP_HIP(do_gather(r, tab, r.sub[0], slot, sc));
      GemmProblem g = weight_gemm(r, /*is_fwd=*/true, j, j + 1, weights_of(r, rep, j, slot), WeightView{nullptr, 0}, X, ldx,
                                  Y, ldy, acc, static_cast<size_t>(j), static_cast<size_t>(n));
      GatherRequest next;
      if (j + 1 < n && !r.dp[j + 1]) {
        next = gather_request(r, tab, r.sub[j + 1], ws + static_cast<size_t>((j + 1) % 2) * r.slot_bytes);
        g.carry = &next;
      }
      g.parts = planes; g.parts_bytes = planes_bytes;
      OSDP_HIP(do_gemm(OSDP_KERNEL_GEMM_FWD, g, sc));
      if (poison && !r.dp[j]) OSDP_HIP(launch_fill16(slot, r.slot_bytes, kPoison, sc));
    }
    return OSDP_OK;
  }
  const bool overlap = two_streams && r.slots == 2 && n > 1 && !pairs;
  hipStream_t sg = overlap ? sp : sc;
  hipEvent_t slot_free[2] = {nullptr, nullptr};  // recorded on the compute stream after the last GEMM that read the slot
  if (overlap) OSDP_HIP(edge(sc, sp));  // the staging area may still be in use by earlier compute-stream work
  for (size_t li = 0; li < r.fwd.size(); ++li) {
    const int j0 = static_cast<int>(r.fwd[li].c0), j1 = static_cast<int>(r.fwd[li].c1);
    void *slot_of[2] = {nullptr, nullptr};
    int slot_id[2] = {0, 0};
    bool gathered = false;
    const bool joint = staged_jointly(r, j0, j1);
    for (int j = j0; j < j1; ++j) {
      const int s = (j1 - j0 == 2) ? j - j0 : j % r.slots;
      slot_id[j - j0] = s;
      slot_of[j - j0] = ws + static_cast<size_t>(s) * r.slot_bytes;
      if (r.dp[j]) continue;  // a DP slice is read where it lies
      if (overlap && slot_free[s]) OSDP_HIP(hipStreamWaitEvent(sp, slot_free[s], 0));  // slot released by its last reader
      if (!joint) OSDP_HIP(do_gather(r, tab, r.sub[j], slot_of[j - j0], sg));
      gathered = true;
    }
    if (joint) OSDP_HIP(do_gather(r, tab, joint_range(r, j0), ws, sg));  // one copy for both, across the two slots
    if (overlap && gathered) OSDP_HIP(edge(sp, sc));
    GemmProblem g =
        joint ? weight_gemm(r, /*is_fwd=*/true, j0, j1, joint_view(r, j0, ws), WeightView{nullptr, 0}, X, ldx, Y, ldy, acc,
                            li, r.fwd.size())
              : weight_gemm(r, /*is_fwd=*/true, j0, j1, weights_of(r, rep, j0, slot_of[0]),
                            weights_of(r, rep, j1 - 1, slot_of[1]), X, ldx, Y, ldy, acc, li, r.fwd.size());
    g.parts = planes; g.parts_bytes = planes_bytes;
    OSDP_HIP(do_gemm(OSDP_KERNEL_GEMM_FWD, g, sc));
    if (poison && gathered) {  // the slices this launch read are dead: poison their slots before they are handed back
      if (joint) OSDP_HIP(launch_fill16(ws, r.slot_bytes * 2, kPoison, sc));
      for (int j = j0; j < j1 && !joint; ++j)
        if (!r.dp[j]) OSDP_HIP(launch_fill16(slot_of[j - j0], r.slot_bytes, kPoison, sc));
    }
    if (overlap && gathered && j1 < n) {
      hipEvent_t ev;
      OSDP_HIP(g_events.get(&ev));
      OSDP_HIP(hipEventRecord(ev, sc));
      for (int j = j0; j < j1; ++j)
        if (!r.dp[j]) slot_free[slot_id[j - j0]] = ev;
    }
  }
  if (overlap) OSDP_HIP(edge(sc, sp));  // later copy-stream work may reuse the workspace
  return OSDP_OK;
}

osdp_status osdp_split_linear_fwd(const osdp_shape *shape, const osdp_plan *plan, int32_t op_index, const void *X,
                                  int64_t ldx, const void *const *w_shards, void *Y, int64_t ldy, void *workspace,
                                  size_t workspace_bytes, void *stream_compute, void *stream_copy) {
  return forward(shape, plan, op_index, false, X, ldx, w_shards, Replicas{nullptr, nullptr, 0}, Y, ldy, workspace,
                 workspace_bytes, stream_compute, stream_copy);
}

// ---- forward without a caller workspace ------------------------------------------------------------------------
// The staging slots (and, for row slices, the fp32 partial sum) live in a fixed array in device memory that is
// part of the library's code object: nothing is allocated, by the library or by the caller.  Every device has
// its own copy of the array at its own address, which is looked up once per device.
constexpr size_t kScratchBytes = OSDP_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {
std::mutex g_scratch_mu;
void *g_scratch_ptr[kEventDevices] = {};  // device address of `scratch` per device, nullptr: not looked up yet

osdp_status scratch_of_current_device(void **out) {
  int dev = 0;
  OSDP_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kEventDevices) return fail(OSDP_ERR_UNSUPPORTED, "device index %d is beyond the %d the library tracks", dev, kEventDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    OSDP_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));  // the address on the device that is current now
    if (!p) return fail(OSDP_ERR_HIP, "hipGetSymbolAddress returned a null address for the scratch array");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return OSDP_OK;
}
}  // namespace

osdp_status osdp_split_linear_fwd_noalloc(const osdp_shape *shape, const osdp_plan *plan, int32_t op_index, const void *X,
                                          int64_t ldx, const void *const *w_shards, void *Y, int64_t ldy, void *stream) {
  // one stream: no events are needed (none is created), and the size is known before anything is enqueued
  Resolved r;
  osdp_status st = resolve(shape, plan, op_index, /*overlap_possible=*/false, /*is_bwd=*/false, &r);
  if (st != OSDP_OK) return st;
  const size_t need = workspace_total(r);
  if (need > kScratchBytes)
    return fail(OSDP_ERR_WORKSPACE,
                "this operator and plan need %zu bytes of staging and partial sums, the built-in scratch array holds %zu: "
                "raise the granularity or use osdp_split_linear_fwd with a workspace",
                need, kScratchBytes);
  void *ws = nullptr;
  if ((st = scratch_of_current_device(&ws)) != OSDP_OK) return st;
  return forward(shape, plan, op_index, false, X, ldx, w_shards, Replicas{nullptr, nullptr, 0}, Y, ldy, ws, kScratchBytes,
                 stream, nullptr);
}

osdp_status osdp_split_linear_fwd_mixed(const osdp_shape *shape, const osdp_plan *plan, int32_t op_index, const void *X,
                                        int64_t ldx, const void *const *w_shards, const void *const *w_dp, int64_t ld_dp,
                                        void *Y, int64_t ldy, void *workspace, size_t workspace_bytes,
                                        void *stream_compute, void *stream_copy) {
  return forward(shape, plan, op_index, true, X, ldx, w_shards, Replicas{w_dp, nullptr, ld_dp}, Y, ldy, workspace,
                 workspace_bytes, stream_compute, stream_copy);
}

static osdp_status backward(const osdp_shape *shape, const osdp_plan *plan, int32_t op_index, bool allow_dp, const void *X,
                            int64_t ldx, const void *dY, int64_t lddy, const void *const *w_shards, const Replicas &rep,
                            void *dX, int64_t lddx, void *const *dw_shards, void *workspace, size_t workspace_bytes,
                            void *stream_compute, void *stream_copy) {
  hipStream_t sc = static_cast<hipStream_t>(stream_compute), sp = static_cast<hipStream_t>(stream_copy);
  const bool two_streams = sp != nullptr && sp != sc;
  Resolved r;
  osdp_status st = resolve(shape, plan, op_index, two_streams, true, &r, allow_dp, &rep);
  if (st != OSDP_OK) return st;
  const bool no_tokens = r.T == 0;  // X, dY and dX have no rows and may be NULL
  if (!no_tokens && (st = check_matrix(X, ldx, r.I, "X")) != OSDP_OK) return st;
  if (!no_tokens && (st = check_matrix(dY, lddy, r.O, "dY")) != OSDP_OK) return st;
  if (!no_tokens && (st = check_matrix(dX, lddx, r.I, "dX")) != OSDP_OK) return st;
  ShardTable tab, gtab;
  if ((st = fill_table(w_shards, r.N, "w_shards", &tab)) != OSDP_OK) return st;
  if ((st = fill_table(reinterpret_cast<const void *const *>(dw_shards), r.N, "dw_shards", &gtab)) != OSDP_OK) return st;
  if ((st = check_replicas(r, rep, true)) != OSDP_OK) return st;
  if ((st = check_workspace(r, workspace, workspace_bytes)) != OSDP_OK) return st;
  if ((st = device_ok()) != OSDP_OK) return st;

  if (no_tokens) {
    // dW = X^T . dY summed over no tokens is zero: the dW launches run with an empty reduction and store the
    // zeros where the gradient belongs; dX is empty, so no weight is gathered.
    for (const Slice &l : r.dw) {
      const GemmProblem gw = dw_gemm(r, static_cast<int>(l.c0), static_cast<int>(l.c1), X, ldx, dY, lddy, gtab, rep);
      OSDP_HIP(do_gemm(OSDP_KERNEL_GEMM_DW, gw, static_cast<hipStream_t>(stream_compute)));
    }
    return OSDP_OK;
  }
  char *ws = static_cast<char *>(workspace);
  float *acc = reinterpret_cast<float *>(ws + r.slot_bytes * r.slots);  // column slices: dX's fp32 partial sum
  void *planes = r.parts_bytes ? ws + r.slot_bytes * r.slots + r.acc_bytes : nullptr;  // row slices: planes of dX launches split along K
  const int n = static_cast<int>(r.sub.size());
  // The gathers of a group run on the copy stream behind dW.  Each group then costs four event operations, which
  // is more than a small gather takes (measured: with 4 MB groups one stream is 5-12 % faster, with 25 MB groups
  // two streams are 1 % faster), so small groups stay on the compute stream.
  // Unless switched off, the gathers of a group do not run as launches of their own at all: the dW launches that
  // precede the group's dX passes need no weights, and take them along (see the forward pass).
  const bool fused = debug_options().fused_gather.load(std::memory_order_relaxed) != 0;
  constexpr double kWorthOverlappingUs = 14.0;
  const bool overlap = !fused && two_streams && r.slots == 2 && n > 1 &&
                       gather_estimate_us(static_cast<int64_t>(r.slot_bytes)) >= kWorthOverlappingUs;  // two slots of slot_bytes / 2 elements
  hipStream_t sg = overlap ? sp : sc;
  hipEvent_t released = nullptr;  // recorded on the compute stream when a group's last GEMM has been enqueued
  const bool poison = debug_options().poison_staging.load(std::memory_order_relaxed) != 0;  // see forward()
  if (poison) OSDP_HIP(launch_fill16(ws, r.slot_bytes * r.slots, kPoison, sc));
  if (overlap) OSDP_HIP(edge(sc, sp));
  size_t next_pass = 0, next_dw = 0;
  for (const Slice &grp : r.group) {
    const int g0 = static_cast<int>(grp.c0), g1 = static_cast<int>(grp.c1);
    // gather every slice of the group into its slot once the previous group has released the slots
    if (overlap && released) OSDP_HIP(hipStreamWaitEvent(sp, released, 0));
    // (a pair of gathered sub-slices that one dX launch will read: one copy, across the two slots)
    const bool joint = staged_jointly(r, g0, g1) && next_pass < r.pass.size() && r.pass[next_pass].c0 == g0 &&
                       r.pass[next_pass].c1 == g1;
    GatherRequest pending[2];
    int n_pending = 0, next_pending = 0;
    if (fused) {
      if (joint) pending[n_pending++] = gather_request(r, tab, joint_range(r, g0), ws);
      for (int j = g0; j < g1 && !joint; ++j)
        if (!r.dp[j]) pending[n_pending++] = gather_request(r, tab, r.sub[j], ws + static_cast<size_t>(j - g0) * r.slot_bytes);
    } else {
      if (joint) OSDP_HIP(do_gather(r, tab, joint_range(r, g0), ws, sg));
      for (int j = g0; j < g1 && !joint; ++j)
        if (!r.dp[j]) OSDP_HIP(do_gather(r, tab, r.sub[j], ws + static_cast<size_t>(j - g0) * r.slot_bytes, sg));
    }
    hipEvent_t gathered = nullptr;
    if (overlap) {
      OSDP_HIP(g_events.get(&gathered));
      OSDP_HIP(hipEventRecord(gathered, sp));
    }
    // dW launches whose range starts in this group: they need no weights and run while the gathers are in flight
    for (; next_dw < r.dw.size() && r.dw[next_dw].c0 < g1; ++next_dw) {
      GemmProblem gw = dw_gemm(r, static_cast<int>(r.dw[next_dw].c0), static_cast<int>(r.dw[next_dw].c1), X, ldx, dY, lddy, gtab, rep);
      if (next_pending < n_pending) gw.carry = &pending[next_pending++];
      OSDP_HIP(do_gemm(OSDP_KERNEL_GEMM_DW, gw, sc));
    }
    for (; next_pending < n_pending; ++next_pending) OSDP_HIP(gather_now(pending[next_pending], sc));  // no dW launch left to take it along
    if (overlap) OSDP_HIP(hipStreamWaitEvent(sc, gathered, 0));
    // the dX launches of the group (column slices: the fp32 partial sum is carried in the workspace between them)
    for (; next_pass < r.pass.size() && r.pass[next_pass].c1 <= g1; ++next_pass) {
      const int j0 = static_cast<int>(r.pass[next_pass].c0), j1 = static_cast<int>(r.pass[next_pass].c1);
      GemmProblem gx =
          joint ? weight_gemm(r, /*is_fwd=*/false, j0, j1, joint_view(r, j0, ws), WeightView{nullptr, 0}, dY, lddy, dX, lddx,
                              acc, next_pass, r.pass.size())
                : weight_gemm(r, /*is_fwd=*/false, j0, j1,
                              weights_of(r, rep, j0, ws + static_cast<size_t>(j0 - g0) * r.slot_bytes),
                              weights_of(r, rep, j1 - 1, ws + static_cast<size_t>(j1 - 1 - g0) * r.slot_bytes), dY, lddy, dX,
                              lddx, acc, next_pass, r.pass.size());
      gx.parts = planes; gx.parts_bytes = r.parts_bytes;
      OSDP_HIP(do_gemm(OSDP_KERNEL_GEMM_DX, gx, sc));
    }
    if (poison) OSDP_HIP(launch_fill16(ws, r.slot_bytes * r.slots, kPoison, sc));
    if (overlap && g1 < n) {
      OSDP_HIP(g_events.get(&released));
      OSDP_HIP(hipEventRecord(released, sc));
    }
  }
  if (overlap) OSDP_HIP(edge(sc, sp));
  return OSDP_OK;
}

osdp_status osdp_split_linear_bwd(const osdp_shape *shape, const osdp_plan *plan, int32_t op_index, const void *X,
                                  int64_t ldx, const void *dY, int64_t lddy, const void *const *w_shards, void *dX,
                                  int64_t lddx, void *const *dw_shards, void *workspace, size_t workspace_bytes,
                                  void *stream_compute, void *stream_copy) {
  return backward(shape, plan, op_index, false, X, ldx, dY, lddy, w_shards, Replicas{nullptr, nullptr, 0}, dX, lddx,
                  dw_shards, workspace, workspace_bytes, stream_compute, stream_copy);
}

osdp_status osdp_split_linear_bwd_mixed(const osdp_shape *shape, const osdp_plan *plan, int32_t op_index, const void *X,
                                        int64_t ldx, const void *dY, int64_t lddy, const void *const *w_shards,
                                        const void *const *w_dp, int64_t ld_dp, void *dX, int64_t lddx,
                                        void *const *dw_shards, void *const *dw_dp, void *workspace,
                                        size_t workspace_bytes, void *stream_compute, void *stream_copy) {
  return backward(shape, plan, op_index, true, X, ldx, dY, lddy, w_shards, Replicas{w_dp, dw_dp, ld_dp}, dX, lddx,
                  dw_shards, workspace, workspace_bytes, stream_compute, stream_copy);
}

osdp_status osdp_granularity_candidates(const osdp_shape *shape, const int32_t *k_list, int32_t n_k,
                                        osdp_granularity_candidate *out, int32_t capacity, int32_t *count) {
  osdp_status st = check_shape(shape);
  if (st != OSDP_OK) return st;
  if (!count) return fail(OSDP_ERR_INVALID_ARG, "count is NULL");
  if (capacity < 0 || (capacity > 0 && !out)) return fail(OSDP_ERR_INVALID_ARG, "out is NULL or capacity negative");
  static const int32_t kDefault[] = {1, 2, 3, 4, 6, 8, 12, 16};
  if (!k_list) {
    k_list = kDefault;
    n_k = static_cast<int32_t>(sizeof kDefault / sizeof kDefault[0]);
  }
  if (n_k <= 0) return fail(OSDP_ERR_INVALID_ARG, "n_k must be positive");
  int32_t n = 0;
  for (int32_t i = 0; i < n_k; ++i) {
    const int32_t k = k_list[i];
    if (k < 1) return fail(OSDP_ERR_INVALID_ARG, "k_list[%d] = %d is below 1", i, k);
    for (uint8_t dim : {uint8_t(OSDP_SPLIT_OUT_FEATURES), uint8_t(OSDP_SPLIT_IN_FEATURES), uint8_t(OSDP_SPLIT_PER_PASS)})
      for (int32_t mode : {int32_t(OSDP_STAGING_SINGLE), int32_t(OSDP_STAGING_DOUBLE), int32_t(OSDP_STAGING_HALF)}) {
        // the unsplit operator is the same execution whichever dimension is named, and has nothing to double-buffer
        if (k == 1 && (mode == OSDP_STAGING_DOUBLE || (mode == OSDP_STAGING_SINGLE && dim != OSDP_SPLIT_OUT_FEATURES))) continue;
        osdp_plan plan = {1, &k, nullptr, mode, &dim};
        Resolved f, b;
        if (resolve(shape, &plan, 0, true, false, &f) != OSDP_OK) continue;  // the kernels do not take this combination
        if (resolve(shape, &plan, 0, true, true, &b) != OSDP_OK) continue;
        if (n < capacity) {
          osdp_granularity_candidate &c = out[n];
          c.k = k; c.staging = mode; c.split_dim = dim; c.reserved = 0;
          c.peak_weight_staging = std::max(f.peak_staging, b.peak_staging);  // (the two passes may cut different dimensions)
          c.workspace = std::max(workspace_total(f), workspace_total(b));
          c.ms = 0.0;
        }
        ++n;
      }
  }
  t_last_error.clear();
  *count = n;
  return OSDP_OK;
}

osdp_status osdp_granularity_select(const osdp_granularity_candidate *cands, int32_t n, size_t staging_budget,
                                    size_t workspace_budget, double max_slowdown, int32_t *chosen) {
  if (!cands || n <= 0) return fail(OSDP_ERR_INVALID_ARG, "no candidates");
  if (!chosen) return fail(OSDP_ERR_INVALID_ARG, "chosen is NULL");
  if (!(max_slowdown >= 0.0)) return fail(OSDP_ERR_INVALID_ARG, "max_slowdown must be >= 0");
  auto fits = [&](const osdp_granularity_candidate &c) {
    return c.ms > 0.0 && (staging_budget == 0 || c.peak_weight_staging <= staging_budget) &&
           (workspace_budget == 0 || c.workspace <= workspace_budget);
  };
  double fastest = -1.0;
  for (int32_t i = 0; i < n; ++i)
    if (fits(cands[i]) && (fastest < 0.0 || cands[i].ms < fastest)) fastest = cands[i].ms;
  if (fastest < 0.0)
    return fail(OSDP_ERR_UNSUPPORTED, "no measured candidate fits the budgets (gathered weights %zu bytes, workspace %zu bytes)",
                staging_budget, workspace_budget);
  const double limit = (1.0 + max_slowdown) * fastest;
  int32_t best = -1;
  for (int32_t i = 0; i < n; ++i) {
    const osdp_granularity_candidate &c = cands[i];
    if (!fits(c) || c.ms > limit) continue;
    if (best < 0 || c.peak_weight_staging < cands[best].peak_weight_staging ||
        (c.peak_weight_staging == cands[best].peak_weight_staging && c.ms < cands[best].ms))
      best = i;
  }
  *chosen = best;
  return OSDP_OK;
}

osdp_status osdp_granularity_measure(const osdp_shape *shape, const void *X, int64_t ldx, const void *dY, int64_t lddy,
                                     const void *const *w_shards, void *Y, int64_t ldy, void *dX, int64_t lddx,
                                     void *const *dw_shards, void *workspace, size_t workspace_bytes, void *stream_compute,
                                     void *stream_copy, osdp_granularity_candidate *cands, int32_t n, int32_t warmup,
                                     int32_t reps) {
  osdp_status st = check_shape(shape);
  if (st != OSDP_OK) return st;
  if (!cands || n <= 0) return fail(OSDP_ERR_INVALID_ARG, "no candidates");
  if (warmup < 0 || reps < 1) return fail(OSDP_ERR_INVALID_ARG, "warmup must be >= 0 and reps >= 1");
  hipStream_t sc = static_cast<hipStream_t>(stream_compute), sp = static_cast<hipStream_t>(stream_copy);
  const bool two_streams = sp != nullptr && sp != sc;
  // everything is checked for every candidate before the first launch
  for (int32_t i = 0; i < n; ++i) {
    const osdp_granularity_candidate &c = cands[i];
    const uint8_t dim = static_cast<uint8_t>(c.split_dim);
    osdp_plan plan = {1, &c.k, nullptr, c.staging, &dim};
    if (c.k < 1 || (c.split_dim != OSDP_SPLIT_OUT_FEATURES && c.split_dim != OSDP_SPLIT_IN_FEATURES && c.split_dim != OSDP_SPLIT_PER_PASS))
      return fail(OSDP_ERR_INVALID_ARG, "candidate %d is malformed", i);
    for (int is_bwd = 0; is_bwd < 2; ++is_bwd) {
      Resolved r;
      if ((st = resolve(shape, &plan, 0, two_streams, is_bwd != 0, &r)) != OSDP_OK) return st;
      if ((st = check_workspace(r, workspace, workspace_bytes)) != OSDP_OK) return st;
    }
  }
  hipEvent_t t0 = nullptr, t1 = nullptr;
  OSDP_HIP(hipEventCreate(&t0));
  hipError_t e = hipEventCreate(&t1);
  if (e != hipSuccess) {
    (void)hipEventDestroy(t0);
    return fail_hip(e, "hipEventCreate");
  }
  st = OSDP_OK;
  for (int32_t i = 0; i < n && st == OSDP_OK; ++i) {
    osdp_granularity_candidate &c = cands[i];
    const uint8_t dim = static_cast<uint8_t>(c.split_dim);
    osdp_plan plan = {1, &c.k, nullptr, c.staging, &dim};
    for (int32_t rep = -warmup; rep < reps && st == OSDP_OK; ++rep) {
      if (rep == 0 && (e = hipEventRecord(t0, sc)) != hipSuccess) st = fail_hip(e, "hipEventRecord");
      if (st == OSDP_OK)
        st = osdp_split_linear_fwd(shape, &plan, 0, X, ldx, w_shards, Y, ldy, workspace, workspace_bytes, stream_compute, stream_copy);
      if (st == OSDP_OK)
        st = osdp_split_linear_bwd(shape, &plan, 0, X, ldx, dY, lddy, w_shards, dX, lddx, dw_shards, workspace,
                                   workspace_bytes, stream_compute, stream_copy);
    }
    if (st != OSDP_OK) break;
    float ms = 0.f;
    if ((e = hipEventRecord(t1, sc)) != hipSuccess || (e = hipEventSynchronize(t1)) != hipSuccess ||
        (e = hipEventElapsedTime(&ms, t0, t1)) != hipSuccess) {
      st = fail_hip(e, "timing a candidate");
      break;
    }
    c.ms = static_cast<double>(ms) / reps;
  }
  (void)hipEventDestroy(t0);
  (void)hipEventDestroy(t1);
  return st;
}

osdp_status osdp_debug_option(const char *name, int32_t value) {
  if (!name) return fail(OSDP_ERR_INVALID_ARG, "option name is NULL");
  for (const DebugSwitch &sw : kSwitches) {
    if (std::strcmp(name, sw.name) != 0) continue;
    if (value < sw.lo || value > sw.hi)
      return fail(OSDP_ERR_INVALID_ARG, "debug option %s takes values %d to %d (got %d)", name, sw.lo, sw.hi, value);
    (debug_options().*sw.field).store(value, std::memory_order_relaxed);
    return OSDP_OK;
  }
  return fail(OSDP_ERR_INVALID_ARG, "unknown debug option %s", name);
}

osdp_status osdp_profile_begin(int32_t max_launches) {
  if (max_launches <= 0) return fail(OSDP_ERR_INVALID_ARG, "max_launches must be positive");
  Profile &pf = t_profile;
  for (TimedLaunch &t : pf.launches) {
    pf.spare.push_back(t.start);
    pf.spare.push_back(t.stop);
  }
  pf.launches.clear();
  pf.carried_launches = 0;
  pf.persistent_launches = 0;
  pf.carried_bytes = 0.0;
  pf.max_launches = static_cast<size_t>(max_launches);
  pf.active = true;
  return OSDP_OK;
}

osdp_status osdp_profile_end(osdp_kernel_stats *stats) {
  Profile &pf = t_profile;
  if (!stats) return fail(OSDP_ERR_INVALID_ARG, "stats is NULL");
  if (!pf.active) return fail(OSDP_ERR_INVALID_ARG, "osdp_profile_begin was not called");
  pf.active = false;
  std::memset(stats, 0, sizeof(osdp_kernel_stats) * OSDP_KERNEL_KINDS);
  OSDP_HIP(hipDeviceSynchronize());
  pf.gemm_iv.clear();
  pf.gather_iv.clear();
  for (TimedLaunch &t : pf.launches) {
    float ms = 0.f, from0 = 0.f;
    OSDP_HIP(hipEventElapsedTime(&ms, t.start, t.stop));
    OSDP_HIP(hipEventElapsedTime(&from0, pf.launches.front().start, t.start));
    (t.kind == OSDP_KERNEL_GATHER ? pf.gather_iv : pf.gemm_iv).push_back({from0, static_cast<double>(from0) + ms});
    osdp_kernel_stats &s = stats[t.kind];
    s.launches += 1;
    s.ms += ms;
    s.flops += t.flops;
    s.bytes += t.bytes;
    pf.spare.push_back(t.start);
    pf.spare.push_back(t.stop);
  }
  pf.launches.clear();
  stats[OSDP_KERNEL_GATHER_CARRIED].launches = pf.carried_launches;
  stats[OSDP_KERNEL_GATHER_CARRIED].bytes = pf.carried_bytes;
  stats[OSDP_KERNEL_GEMM_PERSISTENT].launches = pf.persistent_launches;
  return OSDP_OK;
}

osdp_status osdp_profile_overlap(double *span_ms, double *idle_ms, double *gather_exposed_ms) {
  Profile &pf = t_profile;
  if (pf.active) return fail(OSDP_ERR_INVALID_ARG, "osdp_profile_end has not been called");
  std::vector<std::pair<double, double>> all = pf.gemm_iv, gemm = pf.gemm_iv, gather = pf.gather_iv;
  all.insert(all.end(), gather.begin(), gather.end());
  double lo = 0.0, hi = 0.0;
  for (size_t i = 0; i < all.size(); ++i) {
    lo = i ? std::min(lo, all[i].first) : all[i].first;
    hi = i ? std::max(hi, all[i].second) : all[i].second;
  }
  const double busy = union_length(all), busy_gemm = union_length(gemm);
  if (span_ms) *span_ms = hi - lo;
  if (idle_ms) *idle_ms = (hi - lo) - busy;
  if (gather_exposed_ms) *gather_exposed_ms = busy - busy_gemm;  // time covered by gathers and by no GEMM
  return OSDP_OK;
}

}  // extern "C"
