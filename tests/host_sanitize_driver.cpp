// Driver for the host planners of libcanz under AddressSanitizer / UBSan (CPU only).
// Output arrays are allocated at exactly the sizes include/canz.h documents, so that any
// write past them is caught; results are checked against the invariants the header states.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "canz.h"

static uint64_t g_state = 0x9E3779B97F4A7C15ull;
static uint64_t rnd() {
  g_state ^= g_state << 13, g_state ^= g_state >> 7, g_state ^= g_state << 17;
  return g_state;
}
static int64_t pick(int64_t lo, int64_t hi) { return lo + static_cast<int64_t>(rnd() % static_cast<uint64_t>(hi - lo + 1)); }

#define REQUIRE(cond)                                                      \
  do {                                                                     \
    if (!(cond)) {                                                         \
      std::fprintf(stderr, "case %d: %s failed (line %d): %s\n", iter, #cond, __LINE__, canz_last_error()); \
      return 1;                                                            \
    }                                                                      \
  } while (0)

int main() {
  static const int64_t dims[] = {1, 7, 64, 256, 1024, 4096, 5120, 12288, 25600};
  for (int iter = 0; iter < 3000; ++iter) {
    const int64_t n_buckets = pick(0, 6);
    const int32_t R = static_cast<int32_t>(pick(1, 9));
    std::vector<int64_t> rows, cols, off{0};
    for (int64_t b = 0; b < n_buckets; ++b) {
      const int64_t k = pick(0, 8);
      for (int64_t i = 0; i < k; ++i) rows.push_back(dims[rnd() % 9]), cols.push_back(dims[rnd() % 9]);
      off.push_back(static_cast<int64_t>(rows.size()));
    }
    const int64_t n = static_cast<int64_t>(rows.size());
    std::vector<int64_t> numel(n);
    int64_t total = 0;
    for (int64_t p = 0; p < n; ++p) numel[p] = rows[p] * cols[p], total += numel[p];
    const double alphas[] = {0.0, 0.1, 0.5, 1.0};
    const double alpha = alphas[rnd() % 4];

    std::vector<int64_t> cut(n_buckets * (R + 1)), load(R);
    std::vector<int32_t> owner(n);
    const int32_t kind = rnd() % 2 ? CANZ_COST_NUMEL : CANZ_COST_NS_FLOPS;
    REQUIRE(canz_partition_alpha(n, rows.data(), cols.data(), nullptr, kind, n_buckets, off.data(), R, alpha,
                                 cut.data(), owner.data(), load.data()) == CANZ_OK);
    for (int64_t b = 0; b < n_buckets; ++b) {
      REQUIRE(cut[b * (R + 1)] == 0 && cut[b * (R + 1) + R] == off[b + 1] - off[b]);
      for (int r = 0; r < R; ++r) REQUIRE(cut[b * (R + 1) + r] <= cut[b * (R + 1) + r + 1]);
    }
    for (int64_t p = 0; p < n; ++p) REQUIRE(owner[p] >= 0 && owner[p] < R);

    std::vector<int64_t> nload(R);
    std::vector<int32_t> nowner(n);
    REQUIRE(canz_partition_naive(n, numel.data(), n_buckets, off.data(), R, nowner.data(), nload.data()) == CANZ_OK);
    int64_t sum = 0;
    for (int r = 0; r < R; ++r) sum += nload[r];
    REQUIRE(sum == total);

    // micro-group plan of a random rank: arrays at exactly the owned count
    const int32_t rank = static_cast<int32_t>(pick(0, R - 1));
    int64_t owned = 0;
    for (int64_t p = 0; p < n; ++p) owned += owner[p] == rank;
    std::vector<int32_t> dtype(n, CANZ_DT_BF16);
    std::vector<int64_t> goff(owned + 1), member(owned);
    int64_t n_groups = -1;
    REQUIRE(canz_microgroup_plan(n, rows.data(), cols.data(), dtype.data(), owner.data(), rank,
                                 static_cast<int32_t>(pick(1, 8)), 0, &n_groups, goff.data(), member.data()) == CANZ_OK);
    REQUIRE(n_groups >= 0 && n_groups <= owned && goff[n_groups] == owned);
    for (int64_t i = 0; i < owned; ++i) REQUIRE(member[i] >= 0 && member[i] < n && owner[member[i]] == rank);

    // TP schedule with a capacity just above the largest tensor
    int64_t big = 0;
    for (int64_t p = 0; p < n; ++p) big = numel[p] > big ? numel[p] : big;
    std::vector<int64_t> toff(n + 1), tmem(n), tload(n);
    std::vector<int32_t> thost(n);
    int64_t tg = -1;
    REQUIRE(canz_tp_schedule(n, numel.data(), R, big + pick(0, 1000), &tg, toff.data(), tmem.data(), thost.data(),
                             tload.data()) == CANZ_OK);
    REQUIRE(tg >= 0 && tg <= n && toff[tg] == n);
    std::vector<char> seen(n, 0);
    for (int64_t i = 0; i < n; ++i) {
      REQUIRE(tmem[i] >= 0 && tmem[i] < n && !seen[tmem[i]] && thost[i] >= 0 && thost[i] < R);
      seen[tmem[i]] = 1;
    }
    // error paths must not touch memory either
    if (n > 0) {
      REQUIRE(canz_tp_schedule(n, numel.data(), R, big - 1, &tg, toff.data(), tmem.data(), thost.data(), tload.data()) !=
              CANZ_OK || big == 0);
      REQUIRE(canz_partition_alpha(n, rows.data(), cols.data(), nullptr, kind, n_buckets, off.data(), 0, alpha,
                                   cut.data(), owner.data(), load.data()) == CANZ_EINVAL);
    }
  }
  std::puts("ok");
  return 0;
}
