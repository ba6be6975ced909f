// Host-side rebalancing plan (paper Section 2.3, load balancer paragraph).
// Integer work on a few hundred counters: a few microseconds on one core, so it
// hides behind the static experts' GEMM as the paper intends.  No HIP here.
// Also the macro level of Section 2.3: the Router Predictor's history of routing
// counts and the expert -> rank map derived from it, and the two straggler
// bookkeeping helpers of Section 3.1 (metric, where each expert runs after a plan).
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


// ---------------------------------------------------------------- macro level (Section 2.3)
extern "C" int32_t feplb_history_update(int32_t E, int64_t* hist, const int64_t* n, int32_t shift) {
  FEPLB_REQUIRE(E >= 0 && shift >= 0 && shift <= 30, FEPLB_EINVAL, "history_update: E=%d shift=%d", E, shift);
  FEPLB_REQUIRE((hist && n) || E == 0, FEPLB_EINVAL, "history_update: null array");
  const int64_t div = (int64_t)1 << shift;
  for (int32_t e = 0; e < E; ++e) {
    FEPLB_REQUIRE(n[e] >= 0 && n[e] < ((int64_t)1 << 46), FEPLB_EINVAL, "history_update: n[%d] out of range", e);
    const int64_t diff = (n[e] << FEPLB_HIST_FRAC_BITS) - hist[e];
    int64_t q = diff / div;                       // C++ truncates towards zero;
    if (diff % div != 0 && diff < 0) --q;         // the average is defined with a floor
    hist[e] += q;
  }
  return FEPLB_OK;
}

extern "C" int32_t feplb_place(int32_t P, int32_t E, const int64_t* hist, int32_t cap, const int32_t* owner_in,
                               int32_t* owner_out, int64_t* load_before, int64_t* load_after,
                               int32_t* n_migrated) {
  FEPLB_REQUIRE(P >= 1 && E >= 0 && cap >= 0, FEPLB_EINVAL, "place: bad P/E/cap");
  FEPLB_REQUIRE((hist && owner_in && owner_out) || E == 0, FEPLB_EINVAL, "place: null array");
  FEPLB_REQUIRE((int64_t)cap * P >= E, FEPLB_ESHAPE, "place: %d ranks of %d experts cannot hold %d", P, cap, E);
  std::vector<int64_t> cur(P, 0), load(P, 0);
  for (int32_t e = 0; e < E; ++e) {
    FEPLB_REQUIRE(owner_in[e] >= 0 && owner_in[e] < P, FEPLB_EINVAL, "place: owner_in[%d]=%d", e, owner_in[e]);
    FEPLB_REQUIRE(hist[e] >= 0, FEPLB_EINVAL, "place: hist[%d] negative", e);
    cur[owner_in[e]] += hist[e];
  }
  if (load_before) std::copy(cur.begin(), cur.end(), load_before);
  std::vector<int32_t> order(E), bin_of(E, 0), held(P, 0);
  for (int32_t e = 0; e < E; ++e) order[e] = e;
  std::sort(order.begin(), order.end(), Busier{hist});
  for (int32_t e : order) {
    int32_t best = -1;
    for (int32_t b = 0; b < P; ++b)
      if (held[b] < cap && (best < 0 || load[b] < load[best])) best = b;
    bin_of[e] = best;
    load[best] += hist[e];
    ++held[best];
  }
  const int64_t new_max = E ? *std::max_element(load.begin(), load.end()) : 0;
  const int64_t cur_max = *std::max_element(cur.begin(), cur.end());
  if (E == 0 || new_max >= cur_max) {   // migrating would not lower the predicted maximum: keep the map
    for (int32_t e = 0; e < E; ++e) owner_out[e] = owner_in[e];
    if (load_after) std::copy(cur.begin(), cur.end(), load_after);
    if (n_migrated) *n_migrated = 0;
    return FEPLB_OK;
  }
  // name the bins after ranks so that many experts stay where they are
  std::vector<int32_t> shared((size_t)P * P, 0), rank_of(P, -1);
  std::vector<uint8_t> taken(P, 0);
  for (int32_t e = 0; e < E; ++e) ++shared[(size_t)bin_of[e] * P + owner_in[e]];
  for (int32_t round = 0; round < P; ++round) {
    int32_t pb = -1, pr = -1;
    for (int32_t b = 0; b < P; ++b) {
      if (rank_of[b] >= 0) continue;
      for (int32_t r = 0; r < P; ++r)
        if (!taken[r] && (pb < 0 || shared[(size_t)b * P + r] > shared[(size_t)pb * P + pr])) {
          pb = b;
          pr = r;
        }
    }
    rank_of[pb] = pr;
    taken[pr] = 1;
  }
  std::vector<int64_t> after(P, 0);
  int32_t moved = 0;
  for (int32_t e = 0; e < E; ++e) {
    owner_out[e] = rank_of[bin_of[e]];
    after[owner_out[e]] += hist[e];
    moved += owner_out[e] != owner_in[e];
  }
  if (load_after) std::copy(after.begin(), after.end(), load_after);
  if (n_migrated) *n_migrated = moved;
  return FEPLB_OK;
}

extern "C" int32_t feplb_mark_dynamic(int32_t P, int32_t E, const int32_t* owner, const int64_t* hist,
                                      int32_t dyn, uint8_t* dyn_flag) {
  FEPLB_REQUIRE(P >= 1 && E >= 0 && dyn >= 0, FEPLB_EINVAL, "mark_dynamic: bad P/E/dyn");
  FEPLB_REQUIRE((owner && hist && dyn_flag) || E == 0, FEPLB_EINVAL, "mark_dynamic: null array");
  std::vector<std::vector<int32_t>> mine(P);
  for (int32_t e = 0; e < E; ++e) {
    FEPLB_REQUIRE(owner[e] >= 0 && owner[e] < P, FEPLB_EINVAL, "mark_dynamic: owner[%d]=%d", e, owner[e]);
    mine[owner[e]].push_back(e);
    dyn_flag[e] = 0;
  }
  for (auto& v : mine) {
    std::sort(v.begin(), v.end(), Busier{hist});
    for (size_t i = 0; i < v.size() && i < (size_t)dyn; ++i) dyn_flag[v[i]] = 1;
  }
  return FEPLB_OK;
}

// ---------------------------------------------------------------- straggler bookkeeping (Section 3.1)
extern "C" int32_t feplb_apply_moves(int32_t P, int32_t E, const int32_t* owner, const feplb_move* moves,
                                     int32_t n_moves, int32_t* home) {
  FEPLB_REQUIRE(P >= 1 && E >= 0 && n_moves >= 0, FEPLB_EINVAL, "apply_moves: bad P/E/n_moves");
  FEPLB_REQUIRE((owner && home) || E == 0, FEPLB_EINVAL, "apply_moves: null array");
  FEPLB_REQUIRE(moves || n_moves == 0, FEPLB_EINVAL, "apply_moves: null moves");
  for (int32_t e = 0; e < E; ++e) home[e] = owner[e];
  for (int32_t i = 0; i < n_moves; ++i) {
    FEPLB_REQUIRE(moves[i].expert >= 0 && moves[i].expert < E && moves[i].dst >= 0 && moves[i].dst < P,
                  FEPLB_EINVAL, "apply_moves: move %d names expert %d, rank %d", i, moves[i].expert, moves[i].dst);
    home[moves[i].expert] = moves[i].dst;
  }
  return FEPLB_OK;
}

extern "C" int32_t feplb_straggler(int32_t P, const double* per_rank, double* straggler) {
  FEPLB_REQUIRE(P >= 1 && per_rank && straggler, FEPLB_EINVAL, "straggler: bad arguments");
  double top = per_rank[0], sum = 0.0;
  for (int32_t r = 0; r < P; ++r) {
    top = std::max(top, per_rank[r]);
    sum += per_rank[r];
  }
  *straggler = top - sum / P;
  return FEPLB_OK;
}
