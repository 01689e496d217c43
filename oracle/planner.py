"""Oracle-side FCP planner: atomic sequence grouping and the 2D-DP rank allocator.

TEST INFRASTRUCTURE ONLY; independent of the C++ planner (no shared code, no import).

What the paper fixes (Sec. 4.2 - 4.4, Eq. 2-11, Alg. 1) and the readings taken where it is silent or
at odds with itself:

  * memory (Eq. 7, Cond. 3): a group at degree d must satisfy  sum_k |s_k| * M_token <= (E - M_ms) * d.
    Only the ratio matters, so the planner takes the per-rank capacity in TOKENS,
    cap = floor((E - M_ms) / M_token).  (Eq. 7 prints M_ms inside a group total that is compared with
    E * d; taken literally a d-rank group would hold one copy of the model states.)
  * Stage 1 (Sec. 4.4): sequences in decreasing order of memory (= length; ties keep the input order).
    Each sequence goes into the open bin with the LEAST headroom that still holds it (ties: the bin opened
    first); if none holds it a new bin opens with d_min = ceil(|s| / cap) and capacity d_min * cap.
  * time of a group at degree d (Eq. 8-10).  Eq. 8 as printed has no d, yet Eq. 11 needs T(G, d) and CP
    splits every sequence evenly over the d ranks of its group (Sec. 4.3), so the compute terms are divided by d:
        T_cpa = sum_k alpha1 (1 + eta_k) |s_k|^2 / d          (attention compute)
        T_cp  = T_cpa + sum_k alpha2 |s_k| / d + beta1
        T_cm  = 0 for d = 1, else sum_k alpha3 |s_k| / v + beta2   (Eq. 9; no ring, no exchange)
        T     = T_cp + T_cm - min(T_cpa, T_cma),  T_cma = T_cm      (Eq. 10: all CP traffic is the KV ring)
  * Stage 2 (Eq. 11, Alg. 1): DP[0][0] = 0, everything else +inf;
        DP[i][j] = min over d in [d_min_i, j - sum_{m<i} d_min_m] of max(DP[i-1][j-d], T(G_i, d)),
    the first d that attains the minimum is kept.  Cond. 6 is sum d_p <= N, so the answer is the smallest j <= N
    that attains min_j DP[K'][j] (the text backtracks from DP[K'][N], the listing from one past it; with a
    communication term T need not fall with d, so forcing all N ranks to be used can only hurt).

Plain Python floats (fp64); written for clarity, not speed.
"""
from __future__ import annotations

import itertools
import math
from dataclasses import dataclass

INF = float("inf")


@dataclass(frozen=True)
class CostModel:
    """Coefficients of Eq. 8-9.  alpha3_over_v = alpha3 / v_p (one link speed for every group)."""
    alpha1: float
    alpha2: float
    beta1: float
    alpha3_over_v: float = 0.0
    beta2: float = 0.0


def atomic_groups(seq_lens, cap_tokens):
    """Stage 1 (Sec. 4.4): best-fit-decreasing packing.  Returns (group_of_seq[K], d_min[K'], load[K'])."""
    assert cap_tokens >= 1
    order = sorted(range(len(seq_lens)), key=lambda k: (-int(seq_lens[k]), k))
    group_of = [-1] * len(seq_lens)
    d_min, load = [], []
    for k in order:
        s = int(seq_lens[k])
        assert s >= 1
        best, best_room = -1, None
        for g in range(len(d_min)):
            room = d_min[g] * cap_tokens - load[g]
            if room >= s and (best_room is None or room < best_room):
                best, best_room = g, room
        if best < 0:
            d_min.append(-(-s // cap_tokens))
            load.append(0)
            best = len(d_min) - 1
        load[best] += s
        group_of[k] = best
    return group_of, d_min, load


def group_time(lens, etas, d, cm: CostModel):
    """T(G, d) (Eq. 8-10 with the degree reading of the module docstring)."""
    t_cpa = sum(cm.alpha1 * (1.0 + e) * float(s) * float(s) for s, e in zip(lens, etas)) / d
    t_cp = t_cpa + sum(cm.alpha2 * float(s) for s in lens) / d + cm.beta1
    t_cm = 0.0 if d == 1 else cm.alpha3_over_v * float(sum(lens)) + cm.beta2
    return t_cp + t_cm - min(t_cpa, t_cm)


def allocate(group_lens, group_etas, d_min, n_ranks, cm: CostModel):
    """Stage 2 (Eq. 11, Alg. 1).  Returns (degrees[K'], makespan) or None if sum d_min > N."""
    kp = len(d_min)
    if sum(d_min) > n_ranks:
        return None
    dp = [[INF] * (n_ranks + 1) for _ in range(kp + 1)]
    path = [[0] * (n_ranks + 1) for _ in range(kp + 1)]
    dp[0][0] = 0.0
    for i in range(1, kp + 1):
        before = sum(d_min[:i - 1])
        for j in range(n_ranks + 1):
            for d in range(d_min[i - 1], j - before + 1):
                cost = max(dp[i - 1][j - d], group_time(group_lens[i - 1], group_etas[i - 1], d, cm))
                if cost < dp[i][j]:
                    dp[i][j], path[i][j] = cost, d
    best_j = min(range(n_ranks + 1), key=lambda j: (dp[kp][j], j))
    degrees, j = [0] * kp, best_j
    for i in range(kp, 0, -1):
        degrees[i - 1] = path[i][j]
        j -= path[i][j]
    assert j == 0
    return degrees, dp[kp][best_j]


def allocate_brute_force(group_lens, group_etas, d_min, n_ranks, cm: CostModel):
    """The optimum of Eq. 2 over all degree vectors with d_i >= d_min_i and sum d_i <= N (tiny inputs only)."""
    best = INF
    ranges = [range(dm, n_ranks + 1) for dm in d_min]
    for ds in itertools.product(*ranges):
        if sum(ds) <= n_ranks:
            best = min(best, max((group_time(l, e, d, cm) for l, e, d in zip(group_lens, group_etas, ds)), default=0.0))
    return best


def plan(seq_lens, n_ranks, cap_tokens, cm: CostModel, etas=None):
    """Both stages.  Returns dict(group_of_seq, d_min, degree, base_rank, makespan) or None if infeasible."""
    etas = [0.0] * len(seq_lens) if etas is None else [float(e) for e in etas]
    group_of, d_min, _ = atomic_groups(seq_lens, cap_tokens)
    g_lens = [[] for _ in d_min]
    g_etas = [[] for _ in d_min]
    for k, g in enumerate(group_of):
        g_lens[g].append(int(seq_lens[k]))
        g_etas[g].append(etas[k])
    res = allocate(g_lens, g_etas, d_min, n_ranks, cm)
    if res is None:
        return None
    degrees, makespan = res
    base = [0] * len(degrees)
    for g in range(1, len(degrees)):
        base[g] = base[g - 1] + degrees[g - 1]
    return {"group_of_seq": group_of, "d_min": d_min, "degree": degrees, "base_rank": base, "makespan": makespan}


def group_shard_args(plan_result):
    """Per-sequence (cp_degree, base_rank) when every sequence of an atomic group runs at the group's degree
    (Sec. 4.4: the group is one CP group)."""
    deg = [plan_result["degree"][g] for g in plan_result["group_of_seq"]]
    base = [plan_result["base_rank"][g] for g in plan_result["group_of_seq"]]
    return deg, base
