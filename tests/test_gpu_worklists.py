"""GPU parity for long work lists (micro-batches of many short sequences, the paper's experimental setup packs
hundreds of sequences per batch) and for tensors that are views inside larger allocations."""
import numpy as np
import pytest

import fcp_synth as synth
from oracle import attn as oattn
from oracle import plan as oplan

from parity import TOL_BF16_REL, TOL_LSE_ABS, bf16_tensor_to_f64, check_rank, rel_err

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _many_sequences(n_short, n_sharded, seed):
    rng = np.random.default_rng(seed)
    lens = np.concatenate([rng.integers(1, 41, n_short), rng.integers(30, 200, n_sharded)]).astype(np.int32)
    deg = np.concatenate([np.ones(n_short, np.int32), np.full(n_sharded, 2, np.int32)])
    perm = rng.permutation(len(lens))
    return lens[perm], deg[perm]


def test_work_list_of_1650_items_through_the_plain_entry_points():
    """1500 short sequences and 50 sequences sharded two ways: rank 0 gets 1650 work items (more than the direct
    entry points take, and more than the scheduler's all-pairs overlap scan: every tile then adds with atomics)."""
    lens, deg = _many_sequences(1500, 50, 31)
    wl = synth.custom_workload(lens, deg, hq=4, hkv=2, head_dim=64, seed=32)
    q, k, v, do = synth.draw_qkvdo(wl)
    _, owork = oplan.shard_plan(wl.seq_lens, wl.cp_degree)
    n_items = int((owork["rank"] == 0).sum())
    _say(f"long work list: {len(lens)} sequences, {int(lens.sum())} tokens, {n_items} work items on rank 0")
    assert n_items == 1650
    res = check_rank(wl, q, k, v, do, 0, backward=True, check_partials=False, label="1650 items", direct=False)
    _say("  " + str({a: b for a, b in res.items() if not a.startswith("_")}))


def test_work_list_of_1024_items_through_the_direct_entry_points():
    """The longest list the direct entry points take: 1000 short sequences and 8 sharded ones, 1024 items."""
    lens, deg = _many_sequences(1000, 8, 33)
    wl = synth.custom_workload(lens, deg, hq=4, hkv=2, head_dim=64, seed=34)
    q, k, v, do = synth.draw_qkvdo(wl)
    _, owork = oplan.shard_plan(wl.seq_lens, wl.cp_degree)
    n_items = int((owork["rank"] == 0).sum())
    _say(f"direct work list: {len(lens)} sequences, {int(lens.sum())} tokens, {n_items} work items on rank 0")
    assert n_items == 1024
    res = check_rank(wl, q, k, v, do, 0, backward=True, check_partials=False, label="1024 items")
    _say("  " + str({a: b for a, b in res.items() if not a.startswith("_")}))


def test_work_list_of_300_unsharded_sequences_in_row_order_through_the_direct_entry_points():
    """300 unsharded sequences: one item each, query rows and key ranges ascending with the item number (the
    scheduler finds its sort keys in order and skips the sorts), all rows owned by one unit."""
    rng = np.random.default_rng(35)
    lens = rng.integers(1, 200, 300).astype(np.int32)
    wl = synth.custom_workload(lens, np.ones(300, np.int32), hq=4, hkv=2, head_dim=64, seed=36)
    q, k, v, do = synth.draw_qkvdo(wl)
    _say(f"direct work list in row order: 300 sequences, {int(lens.sum())} tokens")
    res = check_rank(wl, q, k, v, do, 0, backward=True, check_partials=False, label="300 items in row order")
    _say("  " + str({a: b for a, b in res.items() if not a.startswith("_")}))


@pytest.mark.parametrize("family", ["plain", "direct"])
def test_tensors_as_views_inside_larger_buffers_are_not_overrun(family):
    """Every tensor of the call sits inside a larger allocation: the rows after K and V hold NaN, the rows after each
    output hold a sentinel, the last sequence and the last chunk are ragged (not a multiple of any tile).  The
    kernels address tiles through buffer resources that end with the last valid row, so rows past the end must read
    as zero and stores past the end must be dropped: results finite and right, sentinels bit-unchanged."""
    import torch
    from paper_2602_21788_amd.rank import RankAttention
    wl = synth.custom_workload([333, 70, 1, 257, 203], [3, 1, 1, 2, 1], hq=8, hkv=2, head_dim=128, seed=91)
    q, k, v, do = synth.draw_qkvdo(wl)
    ochunks, _ = oplan.shard_plan(wl.seq_lens, wl.cp_degree)
    pad = 300                                            # rows after each tensor (more than any tile)
    for rank in (0, 2):
        ra = RankAttention(wl.seq_lens, wl.cp_degree, rank, wl.hq, wl.hkv, wl.head_dim, wl.softmax_scale)
        ra.set_inputs(q, k, v, do)
        dev = ra.device

        def inside(t, fill):
            big = torch.full((t.shape[0] + pad,) + tuple(t.shape[1:]), fill, dtype=t.dtype, device=dev)
            big[:t.shape[0]].copy_(t)
            return big, big[:t.shape[0]]
        bigs = {}
        for name in ("q", "d_o"):                        # the rank's rows are followed by NaN rows
            bigs[name], view = inside(getattr(ra, name), float("nan"))
            setattr(ra, name, view)
        for name in ("k", "v"):
            bigs[name], view = inside(getattr(ra, name), float("nan"))
            setattr(ra, name, view)
        sentinel = 1024.0
        for name in ("o", "dq", "dk", "dv", "dq_acc", "dk_acc", "dv_acc"):
            bigs[name], view = inside(getattr(ra, name), sentinel)
            setattr(ra, name, view)
        # partial O [n_parts, tq, hq, D]: one padded allocation per slot would change the layout; pad the whole block
        bigs["o_part"] = torch.full((ra.o_part.numel() + pad * wl.hq * wl.head_dim,), sentinel, dtype=torch.float32, device=dev)
        ra.o_part = bigs["o_part"][:ra.o_part.numel()].view(ra.o_part.shape)
        _say(f"views inside larger buffers: {family} entry points, rank {rank}, {ra.tq} rows")
        if family == "plain":
            ra.forward(); ra.backward()
        else:
            ra.forward_direct(); ra.backward_direct()
        torch.cuda.synchronize()
        rows = oplan.rank_rows(ochunks, wl.cu_seqlens, rank)
        O_ref, LSE_ref = oattn.attn_fwd(q, k, v, wl.cu_seqlens, wl.softmax_scale, rows)
        dQ_ref = oattn.attn_dq(q, k, v, do, wl.cu_seqlens, wl.softmax_scale, rows, O_ref, LSE_ref)
        dK_ref, dV_ref = oattn.attn_dkv(q, k, v, do, wl.cu_seqlens, wl.softmax_scale, rows, O_ref, LSE_ref)
        assert np.abs(ra.lse.cpu().numpy().astype(np.float64).T - LSE_ref).max() <= TOL_LSE_ABS
        for name, ref in (("o", O_ref), ("dq", dQ_ref), ("dk", dK_ref), ("dv", dV_ref)):
            got = bf16_tensor_to_f64(getattr(ra, name))
            assert np.isfinite(got).all(), (family, rank, name)
            assert rel_err(got, ref) <= TOL_BF16_REL, (family, rank, name, rel_err(got, ref))
        for name in ("o", "dq", "dk", "dv", "dq_acc", "dk_acc", "dv_acc"):
            tail = bigs[name][getattr(ra, name).shape[0]:]
            assert bool((tail == sentinel).all()), (family, rank, name, "rows after the tensor were written")
        assert bool((bigs["o_part"][ra.o_part.numel():] == sentinel).all()), (family, rank, "o_part overrun")
