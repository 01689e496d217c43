"""Pins of the planner oracle (oracle/planner.py): worked packing example, brute-force optimum of the allocator on
tiny inputs, closed forms and constraints (Sec. 4.2 - 4.4, Eq. 2-11, Alg. 1)."""
import math
import random

import pytest

from oracle import planner as op

CM = op.CostModel(alpha1=2.0e-9, alpha2=3.0e-6, beta1=1.0e-3, alpha3_over_v=4.0e-7, beta2=2.0e-4)
CM_NOCOMM = op.CostModel(alpha1=2.0e-9, alpha2=3.0e-6, beta1=1.0e-3)


def test_bfd_worked_example():
    # capacity 8 tokens per rank; by hand: 10 opens a 2-rank bin (room 6); 7 does not fit it and opens bin 1 (room 1);
    # 5 fits only bin 0 (room 1 left); 4 fits nowhere and opens bin 2 (room 4); 3 goes to bin 2 (room 1);
    # 1 fits all three with room 1 each: the bin opened first takes it.
    group_of, d_min, load = op.atomic_groups([10, 7, 5, 4, 3, 1], 8)
    assert group_of == [0, 1, 0, 2, 2, 0]
    assert d_min == [2, 1, 1] and load == [16, 7, 7]


def test_bfd_prefers_least_headroom_and_keeps_input_order_on_ties():
    # 6 and 6 (same length: the earlier index first) open bins 0 and 1 of capacity 8 (room 2 each); 3 opens bin 2
    # (room 5); 2 fits all, least headroom is 2 (bins 0, 1): bin 0; the next 2 -> bin 1; 1 -> only bin 2 has room.
    group_of, d_min, load = op.atomic_groups([6, 3, 6, 2, 2, 1], 8)
    assert group_of == [0, 2, 1, 0, 1, 2] and d_min == [1, 1, 1] and load == [8, 8, 4]


@pytest.mark.parametrize("seed", range(20))
def test_bfd_invariants(seed):
    rng = random.Random(seed)
    cap = rng.choice([64, 1000, 4096])
    lens = [rng.randint(1, 6 * cap) for _ in range(rng.randint(1, 60))]
    group_of, d_min, load = op.atomic_groups(lens, cap)
    assert sorted(set(group_of)) == list(range(len(d_min)))
    for g, dm in enumerate(d_min):
        members = [lens[k] for k in range(len(lens)) if group_of[k] == g]
        assert sum(members) == load[g] <= dm * cap                      # Cond. 3 at the minimum degree
        assert dm == math.ceil(max(members) / cap)                      # the opener is the longest member
    # no sequence longer than a rank's capacity shares a bin's opener role: every such sequence opened its own bin
    # unless an earlier, longer one had the headroom
    assert sum(d_min) >= math.ceil(sum(lens) / cap)                      # lower bound of any packing


def _random_groups(rng, kp):
    lens, etas, d_min = [], [], []
    for _ in range(kp):
        n = rng.randint(1, 3)
        lens.append([rng.randint(16, 20000) for _ in range(n)])
        etas.append([rng.choice([0.0, 0.0, 0.5, 1.0]) for _ in range(n)])
        d_min.append(rng.randint(1, 2))
    return lens, etas, d_min


@pytest.mark.parametrize("seed", range(60))
def test_dp_equals_brute_force(seed):
    rng = random.Random(1000 + seed)
    kp = rng.randint(1, 6)
    lens, etas, d_min = _random_groups(rng, kp)
    n = rng.randint(1, 8)
    cm = rng.choice([CM, CM_NOCOMM, op.CostModel(1e-9, 0.0, 0.0, 1e-5, 1e-2)])
    res = op.allocate(lens, etas, d_min, n, cm)
    if sum(d_min) > n:
        assert res is None
        return
    degrees, makespan = res
    assert all(d >= dm for d, dm in zip(degrees, d_min)) and sum(degrees) <= n       # Cond. 3 and Cond. 6
    assert makespan == max(op.group_time(l, e, d, cm) for l, e, d in zip(lens, etas, degrees))
    assert makespan == op.allocate_brute_force(lens, etas, d_min, n, cm)                # the optimum of Eq. 2


def test_equal_groups_split_the_ranks_evenly():
    lens = [[4096]] * 4
    etas = [[0.0]] * 4
    degrees, makespan = op.allocate(lens, etas, [1] * 4, 12, CM_NOCOMM)
    assert degrees == [3, 3, 3, 3]
    w = CM_NOCOMM.alpha1 * 4096.0 ** 2 + CM_NOCOMM.alpha2 * 4096.0
    assert makespan == pytest.approx(w / 3 + CM_NOCOMM.beta1, rel=1e-15)


def test_quadratic_cost_sends_ranks_to_the_long_sequence():
    # 16384 costs 16x a 4096 under the quadratic term: with 8 ranks for (16384, 4096, 4096) the optimum gives the long
    # one 6 ranks (16/6 = 2.67 units against 1 unit for the others), not the equal-token split
    cm = op.CostModel(alpha1=1.0, alpha2=0.0, beta1=0.0)
    degrees, makespan = op.allocate([[16384], [4096], [4096]], [[0.0]] * 3, [1, 1, 1], 8, cm)
    assert degrees == [6, 1, 1]
    assert makespan == 16384.0 ** 2 / 6


def test_communication_stops_useless_sharding():
    # a ring costs more than it saves for a short sequence: degree stays 1 although ranks are free (sum d <= N)
    cm = op.CostModel(alpha1=1e-9, alpha2=0.0, beta1=0.0, alpha3_over_v=1e-3, beta2=1.0)
    degrees, makespan = op.allocate([[1024]], [[0.0]], [1], 8, cm)
    assert degrees == [1] and makespan == 1e-9 * 1024.0 ** 2


def test_group_time_overlap_and_degree_one():
    lens, etas = [8192, 1000], [0.0, 1.0]
    t1 = op.group_time(lens, etas, 1, CM)
    assert t1 == (CM.alpha1 * (8192.0 ** 2 + 2 * 1000.0 ** 2) + CM.alpha2 * 9192.0 + CM.beta1)      # no ring, no exchange
    # at degree 2 the exchange (4e-7 * 9192 + 2e-4 = 3.9e-3) hides fully behind the attention compute (6.9e-2):
    t2 = op.group_time(lens, etas, 2, CM)
    assert t2 == pytest.approx((CM.alpha1 * (8192.0 ** 2 + 2 * 1000.0 ** 2) + CM.alpha2 * 9192.0) / 2 + CM.beta1, rel=1e-15)
    # with a slow link the part that exceeds the attention compute shows
    slow = op.CostModel(CM.alpha1, CM.alpha2, CM.beta1, alpha3_over_v=1e-4, beta2=0.0)
    t_cpa = CM.alpha1 * (8192.0 ** 2 + 2 * 1000.0 ** 2) / 2
    assert op.group_time(lens, etas, 2, slow) == pytest.approx(CM.alpha2 * 9192.0 / 2 + CM.beta1 + 1e-4 * 9192.0, rel=1e-15)
    assert 1e-4 * 9192.0 > t_cpa


def test_plan_end_to_end_and_infeasible():
    lens = [30000, 9000, 5000, 3000, 2000, 700, 300, 100]
    res = op.plan(lens, 16, 8192, CM)
    assert res is not None
    assert res["d_min"][res["group_of_seq"][0]] == 4                      # ceil(30000 / 8192)
    assert sum(res["degree"]) <= 16 and all(d >= m for d, m in zip(res["degree"], res["d_min"]))
    assert res["base_rank"] == [sum(res["degree"][:g]) for g in range(len(res["degree"]))]
    assert op.plan(lens, 4, 8192, CM) is None                            # 30000 + 9000 tokens cannot fit 4 ranks: sum d_min > N
