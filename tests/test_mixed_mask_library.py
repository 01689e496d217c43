"""CPU-only checks of the mixed-mask host calls of libfcp.so against the oracle: the shard plan with
full-attention spans and the mask tables are bit-exact (eta to float rounding), and bad span lists are
rejected."""
import ctypes

import numpy as np
import pytest

from oracle import plan as oplan
from paper_2602_21788_amd import binding as B


def _random_spans(rng, lens, density=0.7):
    spans = []
    for k, L in enumerate(lens):
        pos = 0
        while pos < L and rng.random() < density:
            st = pos + int(rng.integers(0, max(2, L // 3)))
            if st >= L:
                break
            ln = min(int(rng.integers(1, max(2, L // 2))), L - st)
            spans.append((k, st, ln))
            pos = st + ln
    return spans


def test_plan_and_tables_bit_exact_random():
    rng = np.random.default_rng(0)
    n_later = 0
    for trial in range(150):
        n = int(rng.integers(1, 5))
        lens = [int(x) for x in rng.integers(1, 120, size=n)]
        deg = [int(x) for x in rng.integers(1, 7, size=n)]
        base = [int(x) for x in rng.integers(0, 4, size=n)] if rng.random() < 0.5 else None
        spans = _random_spans(rng, lens)
        c, w = B.fcp_shard_plan_mixed(lens, deg, spans, base)
        oc, ow = oplan.shard_plan(lens, deg, base, spans=spans)
        assert c.tobytes() == oc.tobytes() and w.tobytes() == ow.tobytes(), (lens, deg, base, spans)
        n_later += int(len(ow) != len(oplan.shard_plan(lens, deg, base)[1]) or
                       ow.tobytes() != oplan.shard_plan(lens, deg, base)[1].tobytes())
        for rank in sorted(set(int(r) for r in oc["rank"])):
            ql, kf, eta = B.fcp_mask_tables(lens, spans, c, rank)
            oql, okf, oeta = oplan.mask_tables(lens, spans, oc, rank)
            assert ql.dtype == np.int32 and ql.tobytes() == oql.tobytes(), (lens, deg, spans, rank)
            assert kf.tobytes() == okf.tobytes()
            np.testing.assert_allclose(eta, oeta, rtol=1e-6, atol=1e-7)
    assert n_later > 20       # the spans did change plans (later chunks became visible) in many trials


def test_no_spans_equals_causal_plan():
    lens, deg = [77, 5, 130], [3, 1, 4]
    c, w = B.fcp_shard_plan_mixed(lens, deg, [])
    c0, w0 = B.fcp_shard_plan(lens, deg)
    assert c.tobytes() == c0.tobytes() and w.tobytes() == w0.tobytes()
    ql, kf, eta = B.fcp_mask_tables(lens, [], c, 0)
    assert (eta == 0).all() and (kf == np.concatenate([np.arange(L) for L in lens])).all()
    mine = c[c["rank"] == 0]
    want = np.concatenate([np.arange(int(x["seq_start"]), int(x["seq_start"]) + int(x["len"])) for x in mine])
    assert (ql == want).all()


def test_eta_feeds_the_group_planner():
    """A sequence that is one big span costs (1 + eta) ~ 2x the causal attention time: with a purely quadratic
    cost the planner gives it about twice the ranks of an equally long causal sequence."""
    lens = [4096, 4096]
    c, _ = B.fcp_shard_plan_mixed(lens, [1, 1], [(0, 0, 4096)])
    _, _, eta = B.fcp_mask_tables(lens, [(0, 0, 4096)], c, 0)
    assert eta[0] == pytest.approx(4095 / 4097, rel=1e-6) and eta[1] == 0
    plan = B.fcp_plan_groups(lens, 12, 4096, (1e-9, 0.0, 0.0, 0.0, 0.0), eta=eta)
    d = plan["degree"][plan["group_of_seq"]]
    assert d[0] == 8 and d[1] == 4


@pytest.mark.parametrize("spans,msg", [
    ([(0, 5, 3), (0, 2, 2)], b"sorted"),            # out of order
    ([(0, 2, 4), (0, 5, 2)], b"overlap"),           # overlapping
    ([(1, 0, 1), (0, 0, 1)], b"sorted"),            # sequences out of order
    ([(0, 8, 3)], b"leaves sequence"),              # past the end
    ([(0, -1, 2)], b"leaves sequence"),
    ([(0, 0, 0)], b"leaves sequence"),              # empty span
    ([(2, 0, 1)], b"out of range"),
])
def test_bad_spans_are_rejected(spans, msg):
    with pytest.raises(B.FcpError) as e:
        B.fcp_shard_plan_mixed([10, 10], [2, 1], spans)
    assert e.value.code == B.FCP_ERR_INVALID_ARG and msg in str(e.value).encode()
    c, _ = B.fcp_shard_plan([10, 10], [2, 1])
    with pytest.raises(B.FcpError):
        B.fcp_mask_tables([10, 10], spans, c, 0)


def test_mask_tables_capacity_and_counts():
    L = B.lib()
    lens = np.array([10, 6], np.int32)
    c, _ = B.fcp_shard_plan(lens, [2, 1])
    nq = ctypes.c_int64(-1)
    rc = L.fcp_mask_tables(lens.ctypes.data, 2, None, 0, c.ctypes.data, len(c), 0, None, 0, ctypes.byref(nq), None, None)
    assert rc == 0 and nq.value == int(c[c["rank"] == 0]["len"].sum())
    small = np.zeros(3, np.int32)
    rc = L.fcp_mask_tables(lens.ctypes.data, 2, None, 0, c.ctypes.data, len(c), 0, small.ctypes.data, 3, ctypes.byref(nq), None, None)
    assert rc == B.FCP_ERR_CAPACITY


def test_mixed_device_entry_points_reject_bad_arguments_on_host():
    L = B.lib()
    fake = ctypes.c_void_p(0x1000)     # never dereferenced: every call below must fail first
    assert L.fcp_attn_fwd_step_mixed(fake, fake, fake, fake, 1, fake, 1, 1, 8, 8, 4, 4, 128, 0.1, None, fake, fake, fake, 1 << 20, None) == B.FCP_ERR_INVALID_ARG
    assert b"q_limit" in L.fcp_last_error()
    assert L.fcp_attn_fwd_step_mixed(fake, fake, fake, fake, 1, fake, 1, 1, 8, 8, 4, 4, 96, 0.1, fake, fake, fake, fake, 1 << 20, None) == B.FCP_ERR_UNSUPPORTED
    assert L.fcp_attn_bwd_step_mixed(fake, fake, fake, fake, fake, fake, fake, 1, fake, 1, 8, 8, 4, 4, 128, 0.1, fake, None, fake, fake, fake, fake, 1 << 20, None) == B.FCP_ERR_INVALID_ARG
    assert L.fcp_attn_bwd_step_mixed(fake, fake, fake, fake, fake, fake, fake, 1, fake, 1, 8, 8, 4, 4, 32, 0.1, fake, fake, fake, fake, fake, fake, 1 << 20, None) == B.FCP_ERR_UNSUPPORTED
