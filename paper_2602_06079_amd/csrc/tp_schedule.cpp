// canz_tp_schedule: micro-group construction with greedy rollback for the TP plane
// (Algorithm 2, Sec. 4.2; Algorithms 3 and 4 in App. C).  Host code.
//
// Tensors in LPT order (cost descending, equal costs by ascending id); a group grows until
// scheduling it onto the host ranks - LPT on a min-heap of (load, rank) - would push the
// largest rank load above the capacity; then the group without the last tensor is final
// and that tensor opens the next group.
#include <algorithm>
#include <functional>
#include <numeric>
#include <queue>
#include <utility>
#include <vector>

#include "canz.h"
#include "canz_internal.h"

namespace {

using Entry = std::pair<int64_t, int32_t>;  // (load, rank), ordered lexicographically

// LPT of `ids` (already in descending cost order) onto n_ranks; returns L_max
int64_t solve(const std::vector<int64_t>& ids, const int64_t* cost, int32_t n_ranks, std::vector<int32_t>* host) {
  std::priority_queue<Entry, std::vector<Entry>, std::greater<Entry>> heap;
  for (int32_t r = 0; r < n_ranks; ++r) heap.push({0, r});
  if (host) host->clear();
  int64_t l_max = 0;
  for (int64_t p : ids) {
    Entry e = heap.top();
    heap.pop();
    if (host) host->push_back(e.second);
    e.first += cost[p];
    l_max = std::max(l_max, e.first);
    heap.push(e);
  }
  return l_max;
}

}  // namespace

extern "C" int canz_tp_schedule(int64_t n_mats, const int64_t* cost, int32_t n_ranks, int64_t cmax,
                                int64_t* n_groups_out, int64_t* group_off_out, int64_t* member_out,
                                int32_t* host_rank_out, int64_t* group_load_out) {
  using canz::fail;
  if (n_mats < 0) return fail(CANZ_EINVAL, "negative n_mats");
  if (!n_groups_out || !group_off_out || (n_mats > 0 && (!member_out || !host_rank_out || !group_load_out)))
    return fail(CANZ_EINVAL, "null output pointer");  // arrays of size zero may be null
  if (n_mats > 0 && !cost) return fail(CANZ_EINVAL, "null cost");
  if (n_ranks < 1) return fail(CANZ_EINVAL, "n_ranks must be >= 1");
  if (cmax < 0) return fail(CANZ_EINVAL, "capacity must be non-negative");
  __int128 total = 0;
  for (int64_t p = 0; p < n_mats; ++p) {
    if (cost[p] < 0) return fail(CANZ_EINVAL, "negative cost at %lld", (long long)p);
    total += cost[p];
  }
  if (total >= (__int128(1) << 62)) return fail(CANZ_EINVAL, "total cost exceeds 2^62");  // rank loads are int64 sums

  std::vector<int64_t> order(n_mats);
  std::iota(order.begin(), order.end(), int64_t(0));
  std::stable_sort(order.begin(), order.end(), [&](int64_t x, int64_t y) { return cost[x] > cost[y]; });

  std::vector<int64_t> current;
  std::vector<int32_t> host;
  int64_t n_groups = 0, n_members = 0;
  group_off_out[0] = 0;
  auto finish = [&]() {
    group_load_out[n_groups] = solve(current, cost, n_ranks, &host);
    for (size_t i = 0; i < current.size(); ++i) {
      member_out[n_members] = current[i];
      host_rank_out[n_members] = host[i];
      ++n_members;
    }
    group_off_out[++n_groups] = n_members;
    current.clear();
  };
  for (int64_t p : order) {
    current.push_back(p);
    if (solve(current, cost, n_ranks, nullptr) <= cmax) continue;
    current.pop_back();  // roll back
    if (current.empty() || cost[p] > cmax)
      return fail(CANZ_ESHAPE, "tensor %lld alone exceeds the capacity", (long long)p);
    finish();
    current.push_back(p);
  }
  if (!current.empty()) finish();
  *n_groups_out = n_groups;
  return CANZ_OK;
}
