"""Pins for the oracle-side shard plan, per-step partials and LSE merge (CPU only).

The chunking rule is this build's reading of the paper's even split over any integer
degree (Sec. 4.2, Sec. 4.3); it is pinned by the worked sizes under tests/golden, by
exact-cover brute force, by a closed form for the per-rank pair count, and by the
algebraic fact that sharded-and-merged attention equals unsharded attention (Eq. 1).
"""
import os

import numpy as np
import pytest

import fcp_synth as synth
from oracle import attn as oattn
from oracle import plan as oplan


def _read_worked(golden_dir):
    out = []
    for line in open(os.path.join(golden_dir, "zigzag_worked_examples.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        a, b, c = [x.strip() for x in line.split("|")]
        L, d = [int(x) for x in a.split()]
        lens = [int(x) for x in b.split()]
        rk, owned, toks = [x.strip() for x in c.split(":")]
        out.append((L, d, lens, int(rk), [int(x) for x in owned.split()], int(toks)))
    return out


def test_worked_examples(golden_dir):
    cases = _read_worked(golden_dir)
    assert len(cases) == 2
    for L, d, lens, rk, owned, toks in cases:
        chunks, work = oplan.shard_plan([L], [d])
        by_chunk = np.sort(chunks, order="chunk")
        assert list(by_chunk["len"]) == lens
        mine = chunks[chunks["rank"] == rk]
        assert sorted(mine["chunk"]) == owned
        assert int(mine["len"].sum()) == toks


def test_case_study_degrees(golden_dir):
    """The plans the paper prints use degrees 1, 2, 3, 4, 6, 8 and 32 ranks each."""
    degrees = set()
    for line in open(os.path.join(golden_dir, "case_study_degrees.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        _, plan = line.split("|")
        tot = 0
        for item in plan.split():
            d, n = [int(x) for x in item.split("x")]
            tot += d * n
            degrees.add(d)
        assert tot == 32
    assert degrees == {1, 2, 3, 4, 6, 8}
    # every such degree yields a valid plan on an awkward length
    for d in sorted(degrees):
        chunks, work = oplan.shard_plan([1000 + d], [d])
        assert int(chunks["len"].sum()) == 1000 + d


@pytest.mark.parametrize("d", range(1, 9))
def test_exact_cover_bruteforce(d):
    """For every L in 1..64: marking each (q, k) pair that some rank's work item makes
    visible covers each causal pair exactly once and nothing above the diagonal."""
    for L in range(1, 65):
        chunks, work = oplan.shard_plan([L], [d])
        assert len(chunks) == (1 if d == 1 else 2 * d)
        assert int(chunks["len"].sum()) == L
        ranks = chunks["rank"]
        assert all((ranks == r).sum() == (1 if d == 1 else 2) for r in range(d))
        mark = np.zeros((L, L), np.int32)
        row_owner = np.full(L, -1)
        for ch in chunks:
            row_owner[ch["seq_start"]:ch["seq_start"] + ch["len"]] = ch["rank"]
        assert (row_owner >= 0).all()
        for w in work:
            assert 0 <= w["step"] < d and w["q_len"] > 0 and w["n_seg"] in (1, 2)
            for qp in range(w["q_seq_start"], w["q_seq_start"] + w["q_len"]):
                assert row_owner[qp] == w["rank"]
                for sgi in range(w["n_seg"]):
                    for kp in range(w["k_seq_start"][sgi], w["k_seq_start"][sgi] + w["k_len"][sgi]):
                        if kp <= qp:
                            mark[qp, kp] += 1
        assert (mark == np.tril(np.ones((L, L), np.int32))).all(), (L, d)
        assert sum(oplan.rank_pairs(work, r) for r in range(d)) == L * (L + 1) // 2


def test_step_owner_rule():
    """Ring step s of group-local rank i reads the chunks owned by rank (i - s) mod d."""
    d, L = 5, 1000
    chunks, work = oplan.shard_plan([L], [d])
    start_to_owner = {int(c["seq_start"]): int(c["rank"]) for c in chunks}
    for w in work:
        for sgi in range(w["n_seg"]):
            assert start_to_owner[int(w["k_seq_start"][sgi])] == (int(w["rank"]) - int(w["step"])) % d


@pytest.mark.parametrize("d,c", [(2, 5), (3, 7), (4, 16), (6, 3), (8, 11)])
def test_balance_closed_form(d, c):
    """When 2d divides L (chunk size c): rank i owns rows [ic, (i+1)c) and
    [(2d-1-i)c, (2d-i)c); summing (position+1) over them gives c^2 (2d-1) + c(c+1)
    visible pairs for every rank -- the zigzag balance."""
    L = 2 * d * c
    _, work = oplan.shard_plan([L], [d])
    for r in range(d):
        assert oplan.rank_pairs(work, r) == c * c * (2 * d - 1) + c * (c + 1)


def test_baseline_pair_counts():
    """Pair counts of the reported ranks of the five workloads (derived independently as
    sums of (position + 1) over the rank's rows)."""
    for cfg, expect_tq in ((0, 512), (1, 1365), (2, 25003), (3, 26214), (4, 24576)):
        wl = synth.make_workload(cfg)
        chunks, work = oplan.shard_plan(wl.seq_lens, wl.cp_degree)
        mine = chunks[chunks["rank"] == wl.rank]
        assert int(mine["len"].sum()) == expect_tq
        direct = sum(int(np.arange(ch["seq_start"] + 1, ch["seq_start"] + ch["len"] + 1, dtype=np.int64).sum())
                     for ch in mine)
        assert oplan.rank_pairs(work, wl.rank) == direct
    wl = synth.make_workload(1)
    _, work = oplan.shard_plan(wl.seq_lens, wl.cp_degree)
    assert [oplan.rank_pairs(work, r) for r in range(3)] == [2794837, 2796202, 2799617]
    r1 = work[work["rank"] == 1]
    per_step = [oplan.rank_pairs(r1[r1["step"] == s], 1) for s in range(3)]
    assert sum(per_step) == 2796202


def test_packed_local_offsets_and_base_rank():
    lens, deg, base = [100, 37, 64, 9], [2, 1, 3, 1], [0, 1, 1, 3]
    chunks, work = oplan.shard_plan(lens, deg, base)
    for r in range(4):
        mine = chunks[chunks["rank"] == r]
        off = 0
        for ch in mine:            # sorted by (seq, chunk): early chunk, then late chunk
            assert ch["local_off"] == off
            off += ch["len"]
    # sequence 2 (degree 3, base 1) lives on ranks 1..3
    assert set(chunks[chunks["seq"] == 2]["rank"]) == {1, 2, 3}
    # order of work items
    keys = [(w["rank"], w["step"], w["seq"], w["q_seq_start"]) for w in work]
    assert keys == sorted(keys)


def test_short_sequence_empty_chunks():
    """L < 2d: the late chunks are empty, still listed, and generate no work."""
    chunks, work = oplan.shard_plan([5], [4])
    assert len(chunks) == 8 and sorted(chunks["len"]) == [0, 0, 0, 1, 1, 1, 1, 1]
    assert (work["q_len"] > 0).all()
    assert sum(oplan.rank_pairs(work, r) for r in range(4)) == 15


@pytest.mark.parametrize("d", range(1, 9))
@pytest.mark.parametrize("L", [17, 100])
def test_sharded_and_merged_equals_unsharded(d, L):
    """Per-step partials over the plan's key sets, merged with ln-sum-exp weights, equal the
    plain definition (Eq. 1, causal) for every degree, power of two or not."""
    wl = synth.custom_workload([L, 23], [d, 1], hq=4, hkv=2, head_dim=8, seed=d * 1000 + L)
    q, k, v, _ = synth.draw_qkvdo(wl)
    cu = wl.cu_seqlens
    O_ref, LSE_ref = oattn.attn_fwd(q, k, v, cu, wl.softmax_scale)
    qf, kf, vf = (synth.bf16_bits_to_f64(x) for x in (q, k, v))
    chunks, work = oplan.shard_plan(wl.seq_lens, wl.cp_degree)
    seen = np.zeros(wl.total_tokens, bool)
    for r in range(d):
        rows = oplan.rank_rows(chunks, cu, r)
        if len(rows) == 0:
            continue
        Op, Lp = oplan.rank_partials(qf, kf, vf, cu, chunks, work, r, wl.softmax_scale)
        O, LSE = oplan.lse_merge(Op, Lp)
        np.testing.assert_allclose(O, O_ref[rows], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(LSE, LSE_ref[rows], rtol=1e-12, atol=1e-12)
        assert not seen[rows].any()
        seen[rows] = True
    assert seen.all()


def test_merge_properties():
    """Merging partials over any partition of the key set gives the whole; the merge is
    order independent; a -inf part is the identity; one part is returned unchanged."""
    rng = np.random.default_rng(11)
    nq, nk, hq, hkv, D = 6, 40, 4, 2, 8
    qf = rng.standard_normal((nq, hq, D)); kf = rng.standard_normal((nk, hkv, D)); vf = rng.standard_normal((nk, hkv, D))
    q_pos = np.full(nq, 10 ** 6); k_pos = np.arange(nk)        # everything visible
    O_all, L_all = oplan.partial_attn(qf, kf, vf, q_pos, k_pos, 0.3)
    cuts = [0, 3, 4, 21, 40]
    parts = [oplan.partial_attn(qf, kf[a:b], vf[a:b], q_pos, k_pos[a:b], 0.3) for a, b in zip(cuts[:-1], cuts[1:])]
    Op = np.stack([p[0] for p in parts]); Lp = np.stack([p[1] for p in parts])
    O, L = oplan.lse_merge(Op, Lp)
    np.testing.assert_allclose(O, O_all, rtol=1e-12, atol=1e-14); np.testing.assert_allclose(L, L_all, rtol=1e-13)
    O2, L2 = oplan.lse_merge(Op[::-1], Lp[::-1])
    np.testing.assert_allclose(O2, O, rtol=1e-13, atol=1e-15); np.testing.assert_allclose(L2, L, rtol=1e-14)
    # two-level merge = flat merge (associativity)
    Oa, La = oplan.lse_merge(Op[:2], Lp[:2]); Ob, Lb = oplan.lse_merge(Op[2:], Lp[2:])
    O3, L3 = oplan.lse_merge(np.stack([Oa, Ob]), np.stack([La, Lb]))
    np.testing.assert_allclose(O3, O, rtol=1e-12, atol=1e-14); np.testing.assert_allclose(L3, L, rtol=1e-13)
    # -inf part: identity, no NaN
    Oi = np.concatenate([Op, np.zeros_like(Op[:1])]); Li = np.concatenate([Lp, np.full_like(Lp[:1], -np.inf)])
    O4, L4 = oplan.lse_merge(Oi, Li)
    np.testing.assert_array_equal(O4, O); np.testing.assert_array_equal(L4, L)
    # single part
    O5, L5 = oplan.lse_merge(Op[:1], Lp[:1])
    np.testing.assert_allclose(O5, Op[0], rtol=1e-15); np.testing.assert_allclose(L5, Lp[0], rtol=1e-15)
    # all parts -inf
    O6, L6 = oplan.lse_merge(np.zeros_like(Op), np.full_like(Lp, -np.inf))
    assert (O6 == 0).all() and np.isneginf(L6).all()


def test_partial_attn_masked_rows():
    """A query placed before every key of the segment sees nothing: O = 0, LSE = -inf."""
    rng = np.random.default_rng(12)
    qf = rng.standard_normal((3, 2, 4)); kf = rng.standard_normal((5, 1, 4)); vf = rng.standard_normal((5, 1, 4))
    O, L = oplan.partial_attn(qf, kf, vf, np.array([0, 7, 100]), np.arange(5, 10), 1.0)
    assert (O[0] == 0).all() and np.isneginf(L[0]).all()
    # the row at position 7 sees keys 5, 6, 7 only
    s = qf[1, 0] @ kf[:3, 0].T
    np.testing.assert_allclose(L[1, 0], np.log(np.exp(s).sum()), rtol=1e-13)
