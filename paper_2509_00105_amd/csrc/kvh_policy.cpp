// Storage policy on the host (Design section of the paper: utility of an entry, marginal utility
// drop, greedy choice per storage tier).  No device code.  An entry's choices are ordered by
// strictly decreasing size (choice 0 = full quality); eviction is the implicit last choice with
// size 0 and utility 0.  Per tier every offered entry starts at its best allowed choice, and
// while the tier is over capacity the step with the smallest marginal utility drop is taken; a
// step may jump from the current choice to any smaller one, which walks the upper convex hull of
// (size, utility) and so reaches the optimum of the linear relaxation up to one fractional step.
// Ties: smaller drop, then lower entry index, then larger remaining size.
#include <cmath>
#include <cstddef>
#include <cstdint>
#include <queue>
#include <vector>

#include "../../include/kvh.h"

static_assert(sizeof(kvh_policy_entry) == 24 && offsetof(kvh_policy_entry, first) == 8 &&
                  offsetof(kvh_policy_entry, n_choices) == 12 && offsetof(kvh_policy_entry, min_choice) == 16,
              "kvh_policy_entry layout");
static_assert(sizeof(kvh_policy_tier) == 16 && offsetof(kvh_policy_tier, capacity) == 8, "kvh_policy_tier layout");

namespace {

constexpr int32_t kEvict = -1;

struct Move {
  double drop;
  int32_t entry;
  double size_after;
  int32_t target;
  int32_t from;  // the choice the move was computed for (stale heap items are skipped)
};
struct Later {
  bool operator()(const Move& a, const Move& b) const {  // true if a comes after b
    if (a.drop != b.drop) return a.drop > b.drop;
    if (a.entry != b.entry) return a.entry > b.entry;
    return a.size_after < b.size_after;
  }
};

inline double utility(double freq, double alpha, double quality, double size, double bandwidth) {
  return freq * (alpha * quality - size / bandwidth);
}
inline double drop_per_byte(double u_m, double u_n, double s_m, double s_n) { return (u_m - u_n) / (s_m - s_n); }

bool integral_size(double s) { return std::isfinite(s) && s > 0.0 && s < 9007199254740992.0 && s == std::floor(s); }

}  // namespace

extern "C" {

double kvh_policy_utility(double freq, double alpha, double quality, double size_bytes, double bandwidth) {
  return utility(freq, alpha, quality, size_bytes, bandwidth);
}

double kvh_policy_marginal_utility_drop(double u_m, double u_n, double size_m, double size_n) {
  return drop_per_byte(u_m, u_n, size_m, size_n);
}

int kvh_policy_plan(const kvh_policy_entry* entries, int n_entries, const double* sizes, const double* qualities,
                    int n_choices_total, const kvh_policy_tier* tiers, int n_tiers, double alpha, int32_t* tier_out,
                    int32_t* choice_out, double* total_utility_out) {
  if (entries == nullptr || sizes == nullptr || qualities == nullptr || tiers == nullptr || tier_out == nullptr ||
      choice_out == nullptr || n_entries < 1 || n_tiers < 1 || n_choices_total < 1 || !std::isfinite(alpha))
    return KVH_E_ARG;
  for (int t = 0; t < n_tiers; ++t)
    if (!(tiers[t].bandwidth > 0.0) || !std::isfinite(tiers[t].bandwidth) || !(tiers[t].capacity >= 0.0)) return KVH_E_ARG;
  double all_sizes = 0.0;  // the sum of the largest choices bounds every occupancy the search can form
  for (int i = 0; i < n_entries; ++i) {
    const kvh_policy_entry& e = entries[i];
    if (e.n_choices < 1 || e.first < 0 || (int64_t)e.first + e.n_choices > n_choices_total) return KVH_E_SHAPE;
    if (e.min_choice < 0 || e.min_choice >= e.n_choices) return KVH_E_SHAPE;
    if (!(e.freq >= 0.0) || !std::isfinite(e.freq)) return KVH_E_ARG;
    for (int j = 0; j < e.n_choices; ++j) {
      if (!integral_size(sizes[e.first + j]) || !std::isfinite(qualities[e.first + j])) return KVH_E_ARG;
      if (j > 0 && !(sizes[e.first + j] < sizes[e.first + j - 1])) return KVH_E_ARG;
    }
    all_sizes += sizes[e.first];
    if (!(all_sizes < 9007199254740992.0)) return KVH_E_SIZE;  // sums would stop being exact
  }

  std::vector<double> u((size_t)n_choices_total);
  std::vector<int32_t> cur((size_t)n_entries);
  std::vector<char> waiting((size_t)n_entries, 1);
  for (int i = 0; i < n_entries; ++i) tier_out[i] = -1, choice_out[i] = kEvict;

  for (int t = 0; t < n_tiers; ++t) {
    const double bandwidth = tiers[t].bandwidth, capacity = tiers[t].capacity;
    double used = 0.0;  // sizes are whole numbers below 2^53: every sum is exact, whatever its order
    auto best_move = [&](int32_t i) {
      const kvh_policy_entry& e = entries[i];
      const double s_m = sizes[e.first + cur[i]], u_m = u[(size_t)e.first + cur[i]];
      Move best{drop_per_byte(u_m, 0.0, s_m, 0.0), i, 0.0, kEvict, cur[i]};
      for (int32_t j = e.n_choices - 1; j > cur[i]; --j) {
        const double s_n = sizes[e.first + j];
        const double d = drop_per_byte(u_m, u[(size_t)e.first + j], s_m, s_n);
        if (d < best.drop || (d == best.drop && s_n > best.size_after)) best = Move{d, i, s_n, j, cur[i]};
      }
      return best;
    };
    std::priority_queue<Move, std::vector<Move>, Later> heap;
    for (int32_t i = 0; i < n_entries; ++i) {
      cur[i] = kEvict;
      if (!waiting[i]) continue;
      const kvh_policy_entry& e = entries[i];
      double best_u = 0.0;
      for (int32_t j = e.min_choice; j < e.n_choices; ++j) {
        const double uj = utility(e.freq, alpha, qualities[e.first + j], sizes[e.first + j], bandwidth);
        u[(size_t)e.first + j] = uj;
        // eviction (utility 0) wins unless a choice is strictly better; among equal choices the smaller stays
        if (uj > best_u || (uj == best_u && cur[i] != kEvict)) cur[i] = j, best_u = uj;
      }
      if (cur[i] != kEvict) {
        used += sizes[e.first + cur[i]];
        heap.push(best_move(i));
      }
    }
    while (used > capacity && !heap.empty()) {
      const Move m = heap.top();
      heap.pop();
      if (cur[m.entry] != m.from) continue;  // computed for a choice the entry has left
      used -= sizes[entries[m.entry].first + cur[m.entry]];
      cur[m.entry] = m.target;
      if (m.target != kEvict) {
        used += m.size_after;
        heap.push(best_move(m.entry));
      }
    }
    for (int32_t i = 0; i < n_entries; ++i)
      if (waiting[i] && cur[i] != kEvict) tier_out[i] = t, choice_out[i] = cur[i], waiting[i] = 0;
  }
  if (total_utility_out != nullptr) {
    double total = 0.0;
    for (int i = 0; i < n_entries; ++i)
      if (tier_out[i] >= 0)
        total += utility(entries[i].freq, alpha, qualities[entries[i].first + choice_out[i]],
                         sizes[entries[i].first + choice_out[i]], tiers[tier_out[i]].bandwidth);
    *total_utility_out = total;
  }
  return KVH_OK;
}

}  // extern "C"
