// canz_microgroup_plan: batch one rank's matrices into same-shape micro-groups.
// Ordering follows the deterministic (cost, id) sort of Algorithm 2, Phase 1, applied to
// shape classes; the byte cap plays the role of C_max.  Host code.
#include <algorithm>
#include <map>
#include <tuple>
#include <vector>

#include "canz.h"
#include "canz_internal.h"

extern "C" int canz_microgroup_plan(int64_t n_mats, const int64_t* rows, const int64_t* cols,
                                    const int32_t* dtype, const int32_t* owner, int32_t rank,
                                    int32_t max_mats, int64_t cmax_bytes, int64_t* n_groups_out,
                                    int64_t* group_off_out, int64_t* member_out) {
  using canz::fail;
  if (n_mats < 0) return fail(CANZ_EINVAL, "negative n_mats");
  if (!n_groups_out || !group_off_out) return fail(CANZ_EINVAL, "null output pointer");
  if (n_mats > 0 && (!rows || !cols || !dtype || !owner)) return fail(CANZ_EINVAL, "null input pointer");
  if (max_mats < 0 || cmax_bytes < 0) return fail(CANZ_EINVAL, "caps must be non-negative");
  int64_t n_owned = 0;
  for (int64_t p = 0; p < n_mats; ++p) {
    if (owner[p] != rank) continue;
    ++n_owned;
    if (rows[p] < 0 || cols[p] < 0 || rows[p] >= (int64_t(1) << 31) || cols[p] >= (int64_t(1) << 31))
      return fail(CANZ_EINVAL, "shape of matrix %lld outside [0, 2^31)", (long long)p);
  }
  if (n_owned > 0 && !member_out) return fail(CANZ_EINVAL, "null output pointer");  // an array of size zero may be null

  using Key = std::tuple<int64_t, int64_t, int32_t>;
  std::map<Key, std::vector<int64_t>> classes;
  for (int64_t p = 0; p < n_mats; ++p)
    if (owner[p] == rank) classes[Key(rows[p], cols[p], dtype[p])].push_back(p);

  struct Cls {
    int64_t numel, first_id;
    const std::vector<int64_t>* ids;
  };
  std::vector<Cls> order;
  for (const auto& kv : classes)
    order.push_back({std::get<0>(kv.first) * std::get<1>(kv.first), kv.second.front(), &kv.second});
  std::sort(order.begin(), order.end(), [](const Cls& x, const Cls& y) {
    return x.numel != y.numel ? x.numel > y.numel : x.first_id < y.first_id;
  });

  int64_t n_groups = 0, n_members = 0;
  group_off_out[0] = 0;
  for (const Cls& c : order) {
    const int64_t one_bytes = 2 * c.numel;
    if (cmax_bytes && one_bytes > cmax_bytes)
      return fail(CANZ_ESHAPE, "matrix %lld alone exceeds cmax_bytes", (long long)c.first_id);
    int64_t in_group = 0;
    for (int64_t p : *c.ids) {
      const bool full = (max_mats && in_group == max_mats) ||
                        (cmax_bytes && static_cast<__int128>(in_group + 1) * one_bytes > cmax_bytes);
      if (in_group > 0 && full) {
        group_off_out[++n_groups] = n_members;
        in_group = 0;
      }
      member_out[n_members++] = p;
      ++in_group;
    }
    if (in_group > 0) group_off_out[++n_groups] = n_members;
  }
  *n_groups_out = n_groups;
  return CANZ_OK;
}
