// canz_partition_alpha: alpha-balanced greedy LPT partitioning (Algorithm 1, Sec. 3.2).
//
// Host code.  Loads are int64; mu, deficits, blend and running target are IEEE fp64 in
// the operation order documented in canz.h.  Build with -ffp-contract=off so that no
// multiply-add is fused: the decisions must be reproducible bit for bit.
#include <algorithm>
#include <cmath>
#include <numeric>
#include <vector>

#include "canz.h"
#include "canz_internal.h"

namespace {

constexpr __int128 LOAD_LIMIT = __int128(1) << 53;  // loads above this are not exact in fp64

// W(p) in 128-bit arithmetic; -1 if it does not stay below LOAD_LIMIT
int64_t checked_cost(int64_t rows, int64_t cols, int cost_kind) {
  const __int128 m = std::min(rows, cols), n = std::max(rows, cols);
  if (n >= (int64_t(1) << 31)) return -1;  // keeps every product below 2^127
  __int128 w;
  if (cost_kind == CANZ_COST_NUMEL) {
    w = m * n;
  } else if (cost_kind == CANZ_COST_NS_FLOPS) {
    w = 5 * (4 * m * m * n + 2 * m * m * m);
  } else if (cost_kind == CANZ_COST_SOAP_FLOPS) {
    // SOAP step, per side of extent d that keeps a basis (d within the limit the model assumes): its share of the
    // rotations of G and M into the bases, of the rotation back and its statistic, 8 r c d; a refresh every 10th
    // step (product 2 d^3, QR 4/3 d^3, accumulation of Q 4/3 d^3): 7/15 d^3 per step; in units of 2^20 FLOPs
    const __int128 lim = CANZ_SOAP_COST_MAX_PRECOND_DIM;
    const __int128 s1 = (m <= lim ? m : 0) + (n <= lim ? n : 0);
    const __int128 s3 = (m <= lim ? m * m * m : 0) + (n <= lim ? n * n * n : 0);
    w = ((120 * m * n * s1 + 7 * s3) / 15) >> 20;
  } else {
    // Shampoo step: statistics and preconditioning products 4 (r^2 c + c^2 r), two inverse roots
    // of 25 rounds x 4 products each: 200 (r^3 + c^3); counted in units of 2^20 FLOPs
    w = (4 * m * n * (m + n) + 200 * (m * m * m + n * n * n)) >> 20;
  }
  return w < LOAD_LIMIT ? static_cast<int64_t>(w) : -1;
}

}  // namespace

extern "C" int canz_partition_alpha(int64_t n_mats, const int64_t* rows, const int64_t* cols,
                                    const int64_t* cost, int32_t cost_kind, int64_t n_buckets,
                                    const int64_t* bucket_off, int32_t n_ranks, double alpha,
                                    int64_t* cut_out, int32_t* owner_out, int64_t* load_out) {
  using canz::fail;
  if (n_mats < 0 || n_buckets < 0) return fail(CANZ_EINVAL, "negative size");
  if (!bucket_off || !load_out || (n_buckets > 0 && !cut_out) || (n_mats > 0 && !owner_out))
    return fail(CANZ_EINVAL, "null pointer");  // arrays of size zero may be null
  if (!cost && (!rows || !cols) && n_mats > 0) return fail(CANZ_EINVAL, "need cost or rows/cols");
  if (n_ranks < 1) return fail(CANZ_EINVAL, "n_ranks must be >= 1");
  if (!(alpha >= 0.0 && alpha <= 1.0)) return fail(CANZ_EINVAL, "alpha must lie in [0,1]");
  if (!cost && cost_kind != CANZ_COST_NUMEL && cost_kind != CANZ_COST_NS_FLOPS && cost_kind != CANZ_COST_SHAMPOO_FLOPS &&
      cost_kind != CANZ_COST_SOAP_FLOPS)
    return fail(CANZ_EUNSUPPORTED, "unknown cost_kind %d", cost_kind);
  if (bucket_off[0] != 0 || bucket_off[n_buckets] != n_mats)
    return fail(CANZ_EINVAL, "bucket_off must run from 0 to n_mats");
  for (int64_t i = 0; i < n_buckets; ++i)
    if (bucket_off[i + 1] < bucket_off[i]) return fail(CANZ_EINVAL, "bucket_off must be non-decreasing");

  // W(p)
  std::vector<int64_t> w(n_mats);
  for (int64_t p = 0; p < n_mats; ++p) {
    if (cost) {
      w[p] = cost[p];
    } else {
      if (rows[p] < 0 || cols[p] < 0) return fail(CANZ_EINVAL, "negative shape at %lld", (long long)p);
      w[p] = checked_cost(rows[p], cols[p], cost_kind);
      if (w[p] < 0) return fail(CANZ_EINVAL, "load of parameter %lld exceeds 2^53", (long long)p);
    }
    if (w[p] < 0) return fail(CANZ_EINVAL, "negative cost at %lld", (long long)p);
    if (w[p] >= LOAD_LIMIT) return fail(CANZ_EINVAL, "load of parameter %lld exceeds 2^53", (long long)p);
  }

  const int R = n_ranks;
  // Phi_i(u): prefix sums per bucket, stored flat at bucket_off[i] + i + u.
  std::vector<int64_t> phi(n_mats + n_buckets);
  std::vector<int64_t> wk(n_buckets);
  int64_t total = 0;
  for (int64_t i = 0; i < n_buckets; ++i) {
    int64_t* ph = phi.data() + bucket_off[i] + i;
    ph[0] = 0;
    const int64_t len = bucket_off[i + 1] - bucket_off[i];
    for (int64_t u = 0; u < len; ++u) {
      // both terms are below 2^53, so the sum cannot wrap before this test trips
      ph[u + 1] = ph[u] + w[bucket_off[i] + u];
      if (ph[u + 1] >= LOAD_LIMIT) return fail(CANZ_EINVAL, "total load exceeds 2^53");
    }
    wk[i] = ph[len];
    total += wk[i];
    if (total >= LOAD_LIMIT) return fail(CANZ_EINVAL, "total load exceeds 2^53");
  }

  std::vector<int64_t> order(n_buckets);
  std::iota(order.begin(), order.end(), int64_t(0));
  std::stable_sort(order.begin(), order.end(), [&](int64_t x, int64_t y) { return wk[x] > wk[y]; });

  std::vector<int64_t> load(R, 0);
  std::vector<double> d(R);
  const double mu = static_cast<double>(total) / static_cast<double>(R);
  const double v_even = 1.0 / static_cast<double>(R);

  for (int64_t t = 0; t < n_buckets; ++t) {
    const int64_t k = order[t];
    const int64_t len = bucket_off[k + 1] - bucket_off[k];
    const int64_t* ph = phi.data() + bucket_off[k] + k;
    int64_t* s = cut_out + k * (int64_t(R) + 1);

    double d_total = 0.0;
    for (int r = 0; r < R; ++r) {
      const double gap = mu - static_cast<double>(load[r]);
      d[r] = gap > 0.0 ? gap : 0.0;
    }
    for (int r = 0; r < R; ++r) d_total = d_total + d[r];

    s[0] = 0;
    double c_run = 0.0;
    for (int r = 0; r + 1 < R; ++r) {
      const double v_fill = d_total > 0.0 ? d[r] / d_total : v_even;
      const double v_star = (1.0 - alpha) * v_even + alpha * v_fill;
      const double target = static_cast<double>(wk[k]) * v_star;
      c_run = c_run + target;
      int64_t best_u = 0;
      double best_gap = std::fabs(static_cast<double>(ph[0]) - c_run);
      for (int64_t u = 1; u <= len; ++u) {
        const double gap = std::fabs(static_cast<double>(ph[u]) - c_run);
        if (gap < best_gap) {
          best_gap = gap;
          best_u = u;
        }
      }
      s[r + 1] = best_u;
      load[r] += ph[s[r + 1]] - ph[s[r]];
    }
    s[R] = len;
    load[R - 1] += ph[s[R]] - ph[s[R - 1]];

    for (int r = 0; r < R; ++r)
      for (int64_t u = s[r]; u < s[r + 1]; ++u) owner_out[bucket_off[k] + u] = r;
  }
  for (int r = 0; r < R; ++r) load_out[r] = load[r];
  return CANZ_OK;
}

// canz_partition_naive: the Atomic Ownership Rule of Sec. 3.1 (Eq. 1) - the static layout
// without load balancing that Algorithm 1 improves on - applied to every bucket on its own
// (App. B.1: each bucket is cut into R equal segments).  With stride S = |B_i| / R, rank r
// owns parameter p iff r S <= Start_Index(p) < (r + 1) S, the start taken inside the bucket.
extern "C" int canz_partition_naive(int64_t n_mats, const int64_t* numel, int64_t n_buckets,
                                    const int64_t* bucket_off, int32_t n_ranks, int32_t* owner_out,
                                    int64_t* load_out) {
  using canz::fail;
  if (n_mats < 0 || n_buckets < 0) return fail(CANZ_EINVAL, "negative size");
  if (!load_out || !bucket_off || (n_mats > 0 && (!numel || !owner_out))) return fail(CANZ_EINVAL, "null pointer");
  if (n_ranks < 1) return fail(CANZ_EINVAL, "n_ranks must be >= 1");
  if (bucket_off[0] != 0 || bucket_off[n_buckets] != n_mats)
    return fail(CANZ_EINVAL, "bucket_off must run from 0 to n_mats");
  for (int64_t i = 0; i < n_buckets; ++i)
    if (bucket_off[i + 1] < bucket_off[i]) return fail(CANZ_EINVAL, "bucket_off must be non-decreasing");
  for (int64_t p = 0; p < n_mats; ++p)
    if (numel[p] < 0) return fail(CANZ_EINVAL, "negative size at %lld", (long long)p);
  for (int r = 0; r < n_ranks; ++r) load_out[r] = 0;
  for (int64_t i = 0; i < n_buckets; ++i) {
    __int128 total = 0, start = 0;
    for (int64_t p = bucket_off[i]; p < bucket_off[i + 1]; ++p) total += numel[p];
    for (int64_t p = bucket_off[i]; p < bucket_off[i + 1]; ++p) {
      // r = floor(start * R / |B_i|), exact in integers
      int64_t r = total > 0 ? static_cast<int64_t>(start * n_ranks / total) : 0;
      r = std::min<int64_t>(r, n_ranks - 1);
      owner_out[p] = static_cast<int32_t>(r);
      load_out[r] += numel[p];
      start += numel[p];
    }
  }
  return CANZ_OK;
}
