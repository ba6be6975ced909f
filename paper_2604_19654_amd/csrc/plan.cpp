// Host-side rebalancing plan (paper Section 2.3, load balancer paragraph).
// Integer work on a few hundred counters: a few microseconds on one core, so it
// hides behind the static experts' GEMM as the paper intends.  No HIP here.
#include <algorithm>
#include <vector>
#include "common.h"

namespace {

struct Busier {
  const int64_t* n;
  bool operator()(int32_t a, int32_t b) const { return n[a] != n[b] ? n[a] > n[b] : a < b; }
};

int32_t receiver_near_half_mean(int32_t P, const std::vector<int64_t>& L, int64_t mean_up) {
  int32_t best = 0;
  auto dist = [&](int32_t r) {
    int64_t v = 2 * L[r] - mean_up;
    return v < 0 ? -v : v;
  };
  for (int32_t r = 1; r < P; ++r)
    if (dist(r) < dist(best)) best = r;
  return best;
}

}  // namespace

extern "C" int32_t feplb_plan(int32_t P, int32_t E, const int32_t* owner, const int64_t* n,
                              const uint8_t* dyn_flag, const int32_t* slots, int64_t tau,
                              int32_t mode, int32_t this_rank, feplb_move* moves,
                              int32_t max_moves, int32_t* n_moves, int64_t* load_before,
                              int64_t* load_after, int32_t* chosen_rank) {
  FEPLB_REQUIRE(P >= 1 && E >= 0 && max_moves >= 0, FEPLB_EINVAL, "plan: bad P/E/max_moves");
  FEPLB_REQUIRE(owner && n && dyn_flag && slots && n_moves, FEPLB_EINVAL, "plan: null input");
  FEPLB_REQUIRE(moves || max_moves == 0, FEPLB_EINVAL, "plan: null moves");
  FEPLB_REQUIRE(mode == FEPLB_PLAN_WHOLE || mode == FEPLB_PLAN_OVERFLOW, FEPLB_EINVAL,
                "plan: unknown mode %d", mode);
  *n_moves = 0;
  std::vector<int64_t> L(P, 0);
  int64_t total = 0;
  for (int32_t e = 0; e < E; ++e) {
    FEPLB_REQUIRE(owner[e] >= 0 && owner[e] < P, FEPLB_EINVAL, "plan: owner[%d]=%d", e, owner[e]);
    FEPLB_REQUIRE(n[e] >= 0, FEPLB_EINVAL, "plan: n[%d] negative", e);
    L[owner[e]] += n[e];
    total += n[e];
  }
  for (int32_t r = 0; r < P; ++r)
    FEPLB_REQUIRE(slots[r] >= 0, FEPLB_EINVAL, "plan: slots[%d] negative", r);
  if (load_before) std::copy(L.begin(), L.end(), load_before);
  int32_t count = 0;

  if (mode == FEPLB_PLAN_WHOLE) {
    if (chosen_rank) *chosen_rank = this_rank;
    const int64_t floor_rows = tau > 1 ? tau : 1;
    // each rank's own eligible experts, busiest first; a cursor-free scan is
    // enough because lists are short (E/P entries).
    std::vector<std::vector<int32_t>> mine(P);
    for (int32_t e = 0; e < E; ++e)
      if (dyn_flag[e] && n[e] >= floor_rows) mine[owner[e]].push_back(e);
    for (auto& v : mine) std::sort(v.begin(), v.end(), Busier{n});
    std::vector<uint8_t> gone(E, 0);
    std::vector<int32_t> room(slots, slots + P);
    for (;;) {
      int32_t src = 0;
      for (int32_t r = 1; r < P; ++r)
        if (L[r] > L[src]) src = r;
      int32_t dst = -1;
      for (int32_t r = 0; r < P; ++r)
        if (r != src && room[r] > 0 && (dst < 0 || L[r] < L[dst])) dst = r;
      if (dst < 0) break;
      int32_t take = -1;
      for (int32_t e : mine[src])
        if (!gone[e] && L[dst] + n[e] < L[src]) {
          take = e;
          break;
        }
      if (take < 0) break;
      FEPLB_REQUIRE(count < max_moves, FEPLB_ECAPACITY, "plan: more than %d moves", max_moves);
      L[src] -= n[take];
      L[dst] += n[take];
      --room[dst];
      gone[take] = 1;
      moves[count++] = feplb_move{take, src, dst, 0, n[take], 0};
    }
  } else {
    const int64_t mean_up = (total + P - 1) / P;
    if (this_rank < 0) this_rank = receiver_near_half_mean(P, L, mean_up);
    FEPLB_REQUIRE(this_rank < P, FEPLB_EINVAL, "plan: this_rank %d out of range", this_rank);
    if (chosen_rank) *chosen_rank = this_rank;
    const int64_t spare = std::max<int64_t>(0, mean_up - L[this_rank]);
    std::vector<int32_t> hot;
    for (int32_t e = 0; e < E; ++e)
      if (dyn_flag[e] && owner[e] != this_rank) hot.push_back(e);
    std::sort(hot.begin(), hot.end(), Busier{n});
    if ((int64_t)hot.size() > slots[this_rank]) hot.resize(slots[this_rank]);
    int64_t hot_rows = 0;
    for (int32_t e : hot) hot_rows += n[e];
    FEPLB_REQUIRE((int32_t)hot.size() <= max_moves, FEPLB_ECAPACITY, "plan: more than %d moves",
                  max_moves);
    for (int32_t e : hot) {
      int64_t rows = 0;
      if (hot_rows > 0) {
        // spare * n[e] stays far below 2^63 for any realistic batch; use a wide
        // product all the same.
        rows = (int64_t)(((__int128)spare * n[e]) / hot_rows);
        rows = std::min(rows, n[e]);
      }
      L[owner[e]] -= rows;
      L[this_rank] += rows;
      moves[count++] = feplb_move{e, owner[e], this_rank, 0, rows, n[e] - rows};
    }
  }
  *n_moves = count;
  if (load_after) std::copy(L.begin(), L.end(), load_after);
  return FEPLB_OK;
}
