// fcp_plan_groups: the FCP scheduler's two stages on the host (paper Sec. 4.4): memory-aware packing of the
// micro-batch's sequences into atomic groups (best-fit decreasing) and the 2D dynamic programme that gives
// every group its CP degree so that the slowest group is as fast as possible (Eq. 2, Eq. 11, Alg. 1), with the
// group time model of Eq. 8-10.  Host only; nothing here touches the GPU.
//
// Readings where the paper is silent or at odds with itself (they are the header's contract):
//   * capacity is given in tokens per rank, (E - M_ms) / M_token: Cond. 3 with Eq. 7 is a ratio of token counts;
//   * the compute terms of Eq. 8 are divided by the degree (Eq. 11 needs T(G, d); CP splits a sequence evenly,
//     Sec. 4.3); a degree-1 group has no ring and no exchange; all CP traffic is the attention's KV ring, so
//     Eq. 10 hides min(attention compute, exchange);
//   * every table entry but DP[0][0] starts at +inf; Cond. 6 is "at most N ranks", so the answer is taken at the
//     smallest rank count that attains the least makespan (with an exchange term more ranks can be slower).
#include <algorithm>
#include <cmath>
#include <limits>
#include <numeric>
#include <vector>

#include "fcp.h"
#include "fcp_internal.h"

namespace {

struct Group {
  std::vector<int32_t> members;   // sequence indices in increasing order
  int64_t load = 0;               // tokens
  int32_t d_min = 0;
  // sums that T(G, d) needs, accumulated in member order
  double quad = 0.0, lin = 0.0, tokens = 0.0;
};

// Eq. 8-10 for one group at degree d
inline double group_time(const Group& g, int d, const fcp_cost_model& cm) {
  const double t_cpa = g.quad / d;
  const double t_cp = t_cpa + g.lin / d + cm.beta1;
  const double t_cm = d == 1 ? 0.0 : cm.alpha3_over_v * g.tokens + cm.beta2;
  return t_cp + t_cm - std::min(t_cpa, t_cm);
}

}  // namespace

extern "C" int fcp_plan_groups(const int32_t* seq_lens, const float* eta, int32_t n_seqs, int32_t n_ranks,
                               int64_t tokens_per_rank, const fcp_cost_model* cm, int32_t* group_of_seq,
                               int32_t* n_groups, int32_t* group_d_min, int32_t* group_degree,
                               int32_t* group_base_rank, double* makespan) {
  using fcp::fail;
  fcp::clear_error();
  if (!seq_lens || !cm || !group_of_seq || !n_groups || !group_d_min || !group_degree || !group_base_rank || !makespan)
    return fail(FCP_ERR_INVALID_ARG, "fcp_plan_groups: null argument");
  if (n_seqs < 0 || n_ranks < 1 || tokens_per_rank < 1)
    return fail(FCP_ERR_INVALID_ARG, "fcp_plan_groups: n_seqs < 0, n_ranks < 1 or tokens_per_rank < 1");
  if (n_ranks > (1 << 16)) return fail(FCP_ERR_UNSUPPORTED, "fcp_plan_groups: more than 65536 ranks");
  for (int32_t k = 0; k < n_seqs; ++k) {
    if (seq_lens[k] < 1) return fail(FCP_ERR_INVALID_ARG, "fcp_plan_groups: seq_lens[%d] = %d < 1", k, seq_lens[k]);
    if (eta && !(eta[k] >= 0.f)) return fail(FCP_ERR_INVALID_ARG, "fcp_plan_groups: eta[%d] negative or NaN", k);
  }
  if (!(cm->alpha1 >= 0.0) || !(cm->alpha2 >= 0.0) || !(cm->beta1 >= 0.0) || !(cm->alpha3_over_v >= 0.0) || !(cm->beta2 >= 0.0))
    return fail(FCP_ERR_INVALID_ARG, "fcp_plan_groups: cost coefficients must be non-negative numbers");

  // ---- Stage 1: best-fit decreasing.  Longest first (equal lengths in input order); a sequence goes to the open
  // group with the least headroom that still holds it (the group opened first among equals), else opens a group
  // of d_min = ceil(len / capacity) ranks.
  std::vector<int32_t> order(n_seqs);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return seq_lens[a] > seq_lens[b]; });
  std::vector<Group> groups;
  for (int32_t k : order) {
    const int64_t s = seq_lens[k];
    int best = -1;
    int64_t best_room = 0;
    for (size_t g = 0; g < groups.size(); ++g) {
      const int64_t room = (int64_t)groups[g].d_min * tokens_per_rank - groups[g].load;
      if (room >= s && (best < 0 || room < best_room)) { best = (int)g; best_room = room; }
    }
    if (best < 0) {
      Group g;
      const int64_t dm = (s + tokens_per_rank - 1) / tokens_per_rank;
      if (dm > n_ranks) {
        *n_groups = 0;
        return fail(FCP_ERR_CAPACITY, "fcp_plan_groups: sequence %d (%d tokens) needs %lld ranks of %lld tokens, %d available",
                    k, seq_lens[k], (long long)dm, (long long)tokens_per_rank, n_ranks);
      }
      g.d_min = (int32_t)dm;
      groups.push_back(g);
      best = (int)groups.size() - 1;
    }
    groups[best].load += s;
    group_of_seq[k] = best;
  }
  const int kp = (int)groups.size();
  *n_groups = kp;
  // members and cost sums in increasing sequence index
  for (int32_t k = 0; k < n_seqs; ++k) {
    Group& g = groups[group_of_seq[k]];
    g.members.push_back(k);
    const double s = (double)seq_lens[k];
    g.quad += cm->alpha1 * (1.0 + (eta ? (double)eta[k] : 0.0)) * s * s;
    g.lin += cm->alpha2 * s;
  }
  int64_t need = 0;
  for (int g = 0; g < kp; ++g) {
    groups[g].tokens = (double)groups[g].load;
    group_d_min[g] = groups[g].d_min;
    need += groups[g].d_min;
  }
  if (need > n_ranks)
    return fail(FCP_ERR_CAPACITY, "fcp_plan_groups: the groups need %lld ranks at their minimum degrees, %d available",
                (long long)need, n_ranks);
  if (kp == 0) {
    *makespan = 0.0;
    return FCP_OK;
  }

  // ---- Stage 2: DP[i][j] = least makespan of the first i groups on exactly j ranks (Eq. 11)
  const double inf = std::numeric_limits<double>::infinity();
  const int N = n_ranks;
  std::vector<double> prev(N + 1, inf), cur(N + 1, inf);
  std::vector<int32_t> path((size_t)kp * (N + 1), 0);
  prev[0] = 0.0;
  int64_t before = 0;                       // sum of d_min of the groups before group i
  std::vector<double> t(N + 1);
  for (int i = 0; i < kp; ++i) {
    const int dm = groups[i].d_min;
    const int d_hi = N - (int)before;       // no j leaves more than this for group i
    for (int d = dm; d <= d_hi; ++d) t[d] = group_time(groups[i], d, *cm);
    std::fill(cur.begin(), cur.end(), inf);
    for (int j = 0; j <= N; ++j)
      for (int d = dm; d <= j - (int)before; ++d) {
        const double cost = std::max(prev[j - d], t[d]);
        if (cost < cur[j]) { cur[j] = cost; path[(size_t)i * (N + 1) + j] = d; }
      }
    before += dm;
    std::swap(prev, cur);
  }
  int best_j = 0;
  for (int j = 1; j <= N; ++j)
    if (prev[j] < prev[best_j]) best_j = j;
  if (!(prev[best_j] < inf)) return fail(FCP_ERR_CAPACITY, "fcp_plan_groups: no feasible allocation found");
  *makespan = prev[best_j];
  int j = best_j;
  for (int i = kp - 1; i >= 0; --i) {
    group_degree[i] = path[(size_t)i * (N + 1) + j];
    j -= group_degree[i];
  }
  int32_t base = 0;
  for (int i = 0; i < kp; ++i) {
    group_base_rank[i] = base;
    base += group_degree[i];
  }
  return FCP_OK;
}

// The paper's atomic groups run as one CP group (Sec. 4.4): every sequence of a group takes the group's degree
// and base rank.
extern "C" int fcp_group_shard_args(const int32_t* group_of_seq, int32_t n_seqs, const int32_t* group_degree,
                                    const int32_t* group_base_rank, int32_t n_groups, int32_t* cp_degree,
                                    int32_t* base_rank) {
  using fcp::fail;
  fcp::clear_error();
  if (n_seqs < 0 || n_groups < 0 || (n_seqs > 0 && (!group_of_seq || !cp_degree || !base_rank)) ||
      (n_groups > 0 && (!group_degree || !group_base_rank)))
    return fail(FCP_ERR_INVALID_ARG, "fcp_group_shard_args: null argument or negative count");
  for (int32_t g = 0; g < n_groups; ++g)
    if (group_degree[g] < 1 || group_base_rank[g] < 0)
      return fail(FCP_ERR_INVALID_ARG, "fcp_group_shard_args: group %d has degree %d, base rank %d", g, group_degree[g],
                  group_base_rank[g]);
  for (int32_t k = 0; k < n_seqs; ++k) {
    const int32_t g = group_of_seq[k];
    if (g < 0 || g >= n_groups)
      return fail(FCP_ERR_INVALID_ARG, "fcp_group_shard_args: group_of_seq[%d] = %d out of range", k, g);
    cp_degree[k] = group_degree[g];
    base_rank[k] = group_base_rank[g];
  }
  return FCP_OK;
}
