"""fcp_plan_groups (C ABI, host C++) against the planner oracle: groups, minimum degrees, degrees and base ranks
bit-exact; makespan to 1e-12 relative (same arithmetic, fp64).  Plus the error paths and the solver's time on a
micro-batch of the size the paper reports scheduling times for (Sec. 6, scheduling overhead)."""
import random
import time

import numpy as np
import pytest

import fcp_synth as synth
import paper_2602_21788_amd as fcp
from oracle import planner as op
from paper_2602_21788_amd import binding as B

CMS = [(2.0e-9, 3.0e-6, 1.0e-3, 4.0e-7, 2.0e-4), (2.0e-9, 3.0e-6, 1.0e-3, 0.0, 0.0), (1e-9, 0.0, 0.0, 1e-5, 1e-2)]


def _compare(lens, n_ranks, cap, cm, eta=None):
    eta32 = None if eta is None else np.asarray(eta, np.float32)
    ref = op.plan(lens, n_ranks, cap, op.CostModel(*cm), None if eta32 is None else [float(e) for e in eta32])
    if ref is None:
        with pytest.raises(fcp.FcpError) as ei:
            fcp.fcp_plan_groups(lens, n_ranks, cap, cm, eta32)
        assert ei.value.code == B.FCP_ERR_CAPACITY
        return None
    got = fcp.fcp_plan_groups(lens, n_ranks, cap, cm, eta32)
    assert got["group_of_seq"].tolist() == ref["group_of_seq"]
    assert got["d_min"].tolist() == ref["d_min"]
    assert got["degree"].tolist() == ref["degree"]
    assert got["base_rank"].tolist() == ref["base_rank"]
    assert got["makespan"] == pytest.approx(ref["makespan"], rel=1e-12, abs=0.0)
    return got


@pytest.mark.parametrize("seed", range(80))
def test_random_micro_batches(seed):
    rng = random.Random(seed)
    cap = rng.choice([512, 4096, 8192])
    k = rng.randint(0, 40)
    lens = [max(1, int(rng.lognormvariate(6.5, 1.3))) for _ in range(k)]
    eta = None if seed % 3 else [rng.choice([0.0, 0.25, 1.0]) for _ in range(k)]
    n_ranks = rng.randint(1, 40)
    _compare(lens, n_ranks, cap, CMS[seed % 3], eta)


def test_bench_workloads():
    for cfg in range(5):
        wl = synth.make_workload(cfg)
        _compare(wl.seq_lens.tolist(), 8, 8192, CMS[0])
        _compare(wl.seq_lens.tolist(), 32, 4096, CMS[2])


def test_ties_and_edges():
    _compare([6, 3, 6, 2, 2, 1], 4, 8, CMS[1])              # equal lengths, equal headrooms
    _compare([10, 7, 5, 4, 3, 1], 5, 8, CMS[0])
    _compare([1], 1, 1, CMS[0])
    _compare([], 3, 100, CMS[0])                           # empty micro-batch: no groups, makespan 0
    _compare([4096] * 4, 12, 4096, CMS[1])                 # equal groups: 3 ranks each
    _compare([100000], 8, 4096, CMS[0])                    # needs 25 ranks: infeasible
    got = fcp.fcp_plan_groups([], 3, 100, CMS[0])
    assert len(got["degree"]) == 0 and got["makespan"] == 0.0


def test_invalid_arguments():
    for bad in (dict(lens=[0, 5]), dict(n_ranks=0), dict(cap=0), dict(cm=(-1.0, 0, 0, 0, 0)), dict(eta=[-0.5, 0.0])):
        kw = dict(lens=[8, 5], n_ranks=4, cap=16, cm=CMS[0], eta=None)
        kw.update(bad)
        with pytest.raises(fcp.FcpError) as ei:
            fcp.fcp_plan_groups(kw["lens"], kw["n_ranks"], kw["cap"], kw["cm"], kw["eta"])
        assert ei.value.code == B.FCP_ERR_INVALID_ARG


def test_solver_time_large_micro_batch():
    """512 sequences on 64 ranks (the paper's largest reported setting: solver time below 86 ms there)."""
    rng = np.random.default_rng(7)
    lens = np.clip(rng.lognormal(6.5, 1.2, 512), 64, 32768).astype(np.int32)
    t0 = time.perf_counter()
    got = fcp.fcp_plan_groups(lens, 64, 16384, CMS[0])
    dt = time.perf_counter() - t0
    print(f"fcp_plan_groups: 512 sequences, 64 ranks -> {len(got['degree'])} groups in {dt * 1e3:.2f} ms")
    assert sum(got["degree"]) <= 64 and dt < 0.086


def test_profiler_fit_recovers_coefficients():
    from paper_2602_21788_amd import profiler
    rng = np.random.default_rng(3)
    lens = rng.integers(256, 32768, 24).astype(np.float64)
    deg = rng.integers(1, 8, 24).astype(np.float64)
    a1, a2, b1 = 2.5e-10, 4.0e-7, 3.0e-4
    t = a1 * lens ** 2 / deg + a2 * lens / deg + b1
    (f1, f2, fb), err = profiler.fit_compute_coefficients(lens, deg, t)
    assert f1 == pytest.approx(a1, rel=1e-6) and f2 == pytest.approx(a2, rel=1e-6) and fb == pytest.approx(b1, rel=1e-6)
    assert err < 1e-9
    noisy = t * (1 + 0.03 * rng.standard_normal(24))
    (g1, _, _), _ = profiler.fit_compute_coefficients(lens, deg, noisy)
    assert g1 == pytest.approx(a1, rel=0.1)          # the quadratic term dominates and survives 3 % noise


def test_group_shard_args_and_rank_coverage():
    """Every sequence takes its group's degree and base rank (the paper's atomic groups); the shard plan built from them
    places every token on exactly one rank of its group, and no rank holds more tokens than its budget allows."""
    from oracle import plan as oplan
    rng = np.random.default_rng(11)
    for trial in range(30):
        lens = [int(x) for x in rng.integers(16, 9000, size=int(rng.integers(1, 12)))]
        n_ranks, cap = 16, 4096
        cm = (1e-9, 1e-6, 1e-4, 2e-7, 1e-4)
        try:
            plan = B.fcp_plan_groups(lens, n_ranks, cap, cm)
        except B.FcpError:
            continue
        oplan_res = op.plan(lens, n_ranks, cap, op.CostModel(*cm))
        deg, base = B.fcp_group_shard_args(plan["group_of_seq"], plan["degree"], plan["base_rank"])
        odeg, obase = op.group_shard_args(oplan_res)
        assert list(deg) == odeg and list(base) == obase
        chunks, _ = B.fcp_shard_plan(lens, deg, base)
        per_rank = np.zeros(n_ranks, np.int64)
        for c in chunks:
            g = plan["group_of_seq"][c["seq"]]
            assert plan["base_rank"][g] <= c["rank"] < plan["base_rank"][g] + plan["degree"][g]
            per_rank[c["rank"]] += c["len"]
        assert per_rank.sum() == sum(lens)
        # an even split of every sequence of a group over its d ranks: at most ceil-rounding above load / d,
        # one token per chunk pair and sequence
        for g in range(len(plan["degree"])):
            seqs = [k for k in range(len(lens)) if plan["group_of_seq"][k] == g]
            load, d = sum(lens[k] for k in seqs), int(plan["degree"][g])
            ranks = per_rank[plan["base_rank"][g]: plan["base_rank"][g] + d]
            assert ranks.max() <= load / d + 2 * len(seqs) and ranks.max() <= cap + 2 * len(seqs)
    with pytest.raises(B.FcpError):
        B.fcp_group_shard_args([0, 2], [1, 1], [0, 1])
