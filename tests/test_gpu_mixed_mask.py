"""GPU parity under mixed masks (full attention inside marked spans, causal elsewhere): the HIP path through
fcp_shard_plan_mixed / fcp_mask_tables / fcp_attn_*_step_mixed against the fp64 oracle, element by element.
The spans are placed to cross tile borders of every kernel (32 / 64 / 128 / 256 rows or keys), chunk borders of
the zigzag split, and sequence ends."""
import numpy as np
import pytest

import fcp_synth as synth
from oracle import attn as oattn
from oracle import plan as oplan

from parity import TOL_BF16_REL, check_rank, rel_err

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _show(res):
    return {a: b for a, b in res.items() if not a.startswith("_")}


@pytest.mark.parametrize("D", [128, 64])
def test_single_sequence_spans_across_tile_borders(D):
    L = 1000
    spans = [(0, 10, 5), (0, 100, 300), (0, 450, 64), (0, 600, 130), (0, 900, 100)]
    wl = synth.custom_workload([L], [1], hq=4, hkv=2, head_dim=D, seed=31)
    q, k, v, do = synth.draw_qkvdo(wl)
    _say(f"mixed mask: L={L} d=1 D={D} spans {spans}")
    res = check_rank(wl, q, k, v, do, 0, backward=True, check_partials=True, label=f"mixed-single-D{D}", spans=spans)
    _say(f"  {_show(res)}")


def test_whole_sequence_span_is_bidirectional():
    """Every token sees every token: each query tile runs over all keys, each key tile over all rows."""
    lens = [700, 129]
    spans = [(0, 0, 700), (1, 0, 129)]
    wl = synth.custom_workload(lens, [1, 1], hq=8, hkv=2, head_dim=128, seed=32)
    q, k, v, do = synth.draw_qkvdo(wl)
    _say("mixed mask: whole-sequence spans")
    res = check_rank(wl, q, k, v, do, 0, backward=True, check_partials=True, label="mixed-full", spans=spans)
    _say(f"  {_show(res)}")


@pytest.mark.parametrize("d", [2, 3, 5])
def test_spans_across_chunk_borders_all_ranks(d):
    """A sharded sequence whose spans cross the zigzag chunk borders (so later key chunks become visible), packed
    with a short degree-1 sequence that has a span of its own; every rank is checked and the ranks' dK/dV add up
    to the unsharded gradient."""
    L = 1531 + 7 * d
    bounds = oplan.chunk_bounds(L, d)
    spans = []
    for c in range(1, len(bounds), 2):                      # a span over every second chunk border
        b = bounds[c][0]
        spans.append((0, b - 37, 90))
    spans.append((0, L - 20, 20))
    spans.append((1, 3, 50))
    wl = synth.custom_workload([L, 75], [d, 1], hq=4, hkv=2, head_dim=128, seed=40 + d)
    q, k, v, do = synth.draw_qkvdo(wl)
    sid = oplan.span_ids(wl.seq_lens, spans)
    causal_items = len(oplan.shard_plan(wl.seq_lens, wl.cp_degree)[1])
    mixed_items = oplan.shard_plan(wl.seq_lens, wl.cp_degree, spans=spans)[1]
    assert len(mixed_items) > causal_items or (mixed_items["n_seg"] == 2).sum() > 0
    dK_sum = dV_sum = None
    for r in range(d):
        _say(f"mixed mask: degree {d} rank {r} L={L}")
        res = check_rank(wl, q, k, v, do, r, backward=True, check_partials=True, label=f"mixed-d{d}r{r}", spans=spans)
        dK_sum = res["_dK_acc"] if dK_sum is None else dK_sum + res["_dK_acc"]
        dV_sum = res["_dV_acc"] if dV_sum is None else dV_sum + res["_dV_acc"]
    _, dK_ref, dV_ref = oattn.attn_bwd(q, k, v, do, wl.cu_seqlens, wl.softmax_scale, span_id=sid)
    assert rel_err(dK_sum, dK_ref) <= TOL_BF16_REL and rel_err(dV_sum, dV_ref) <= TOL_BF16_REL


def test_many_short_sequences_random_spans():
    rng = np.random.default_rng(6)
    lens = [int(x) for x in rng.integers(1, 300, size=30)]
    spans = []
    for kk, L in enumerate(lens):
        pos = 0
        while pos < L and rng.random() < 0.7:
            st = pos + int(rng.integers(0, max(2, L // 3)))
            if st >= L:
                break
            ln = min(int(rng.integers(1, max(2, L // 2))), L - st)
            spans.append((kk, st, ln))
            pos = st + ln
    wl = synth.custom_workload(lens, np.ones(30, np.int32), hq=6, hkv=2, head_dim=64, seed=33)
    q, k, v, do = synth.draw_qkvdo(wl)
    _say(f"mixed mask: 30 short sequences, {len(spans)} random spans")
    res = check_rank(wl, q, k, v, do, 0, backward=True, check_partials=True, label="mixed-shorts", spans=spans)
    _say(f"  {_show(res)}")


def test_empty_span_list_equals_causal_entry_points():
    """The mixed entry points with tables of a span-free mask give the causal entry points' result bit for bit."""
    import torch
    from paper_2602_21788_amd.rank import RankAttention
    wl = synth.custom_workload([517, 300], [2, 1], hq=4, hkv=2, head_dim=128, seed=34)
    q, k, v, do = synth.draw_qkvdo(wl)
    outs = []
    for spans in (None, []):
        ra = RankAttention(wl.seq_lens, wl.cp_degree, 0, wl.hq, wl.hkv, wl.head_dim, wl.softmax_scale, spans=spans)
        ra.set_inputs(q, k, v, do)
        ra.forward(); ra.backward()
        torch.cuda.synchronize()
        outs.append([x.clone() for x in (ra.o, ra.lse, ra.dq, ra.dk, ra.dv)])
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_cfg2_image_spans_full_size_sampled():
    """The 32K-token packed workload with its synthetic image spans, in the launch configuration `bench.py --mask
    mixed` times (rank 0, 32 query / 8 KV heads, D = 128): O, LSE, dQ of every 61st row and dK, dV in full for the
    query heads of KV head 3 (heads are independent, so a head subset is exact for those heads)."""
    import torch
    from paper_2602_21788_amd.rank import RankAttention
    from parity import TOL_LSE_ABS, bf16_tensor_to_f64
    wl = synth.make_workload(2)
    spans = synth.image_spans(wl.seq_lens, wl.seed)
    sid = oplan.span_ids(wl.seq_lens, spans)
    q, k, v, do = synth.draw_qkvdo(wl)
    _say(f"cfg2 {wl.name} + {len(spans)} image spans, rank {wl.rank}: full-size run, sampled comparison")
    ra = RankAttention(wl.seq_lens, wl.cp_degree, wl.rank, wl.hq, wl.hkv, wl.head_dim, wl.softmax_scale, spans=spans)
    ra.set_inputs(q, k, v, do)
    ra.forward()
    ra.backward()
    torch.cuda.synchronize()
    ochunks, _ = oplan.shard_plan(wl.seq_lens, wl.cp_degree, spans=spans)
    rows = oplan.rank_rows(ochunks, wl.cu_seqlens, wl.rank)
    O = bf16_tensor_to_f64(ra.o)
    LSE = ra.lse.cpu().numpy().astype(np.float64).T
    dQ, dK, dV = (bf16_tensor_to_f64(x) for x in (ra.dq, ra.dk, ra.dv))
    for x in (O, LSE, dQ, dK, dV):
        assert np.isfinite(x).all()
    G, kvh = wl.hq // wl.hkv, 3
    sel = np.arange(0, len(rows), 61)
    hs = slice(kvh * G, (kvh + 1) * G)
    qs, dos = np.ascontiguousarray(q[:, hs]), np.ascontiguousarray(do[:, hs])
    ks, vs = np.ascontiguousarray(k[:, kvh:kvh + 1]), np.ascontiguousarray(v[:, kvh:kvh + 1])
    O_ref, LSE_ref = oattn.attn_fwd(qs, ks, vs, wl.cu_seqlens, wl.softmax_scale, rows, span_id=sid)
    dQ_ref = oattn.attn_dq(qs, ks, vs, dos, wl.cu_seqlens, wl.softmax_scale, rows[sel], O_ref[sel], LSE_ref[sel], span_id=sid)
    dK_ref, dV_ref = oattn.attn_dkv(qs, ks, vs, dos, wl.cu_seqlens, wl.softmax_scale, rows, O_ref, LSE_ref, span_id=sid)
    e = {"O": rel_err(O[sel, hs], O_ref[sel]), "LSE": float(np.abs(LSE[sel, hs] - LSE_ref[sel]).max()),
         "dQ": rel_err(dQ[sel, hs], dQ_ref), "dK": rel_err(dK[:, kvh:kvh + 1], dK_ref), "dV": rel_err(dV[:, kvh:kvh + 1], dV_ref)}
    _say(f"  kv head {kvh}: {e}")
    assert e["LSE"] <= TOL_LSE_ABS and all(e[n] <= TOL_BF16_REL for n in ("O", "dQ", "dK", "dV"))
    # the image spans did matter: the causal result of the same inputs differs
    O_c, _ = oattn.attn_fwd(qs, ks, vs, wl.cu_seqlens, wl.softmax_scale, rows[sel])
    assert rel_err(O_c, O_ref[sel]) > 0.05
