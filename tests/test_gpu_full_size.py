"""GPU parity at full size: the large workloads, in the launch configuration bench.py times, through BOTH families of
entry points (plain: partial results + merge, fp32 accumulators + finalize; direct), each compared WITH THE ORACLE.

The fp64 oracle cannot redo a 131072-token sequence in seconds, so per workload and KV-head group (heads are
independent: a head subset is the exact result for those heads):
  dense run (the benchmark's inputs)
    - O, LSE, dQ of every `stride`-th row of the rank (stride < 32, so every 32-row block of every tile is hit);
    - dK, dV of the last keys of the rank's last chunk (only the few rows after them see those keys), all their
      rows included;
    - two identities that hold at any size, over ALL keys of the pool in fp64: sum_j dV_j = sum of dO over the
      rank's rows and the group's heads (every row's probabilities add up to 1), and sum_j dK_j = 0 (every row
      of dS adds up to 0);
  sparse run: dO is zero except on the sampled rows.  Rows with dO = 0 contribute exactly nothing to any gradient
    (dP = 0 and delta = 0, so dS = 0, and P^T dO = 0), so dK and dV of EVERY pool key are the sums over the sampled
    rows alone, which the oracle can form; the kernels still run every tile of the full-size launch.
"""
import numpy as np
import pytest

import fcp_synth as synth
from oracle import attn as oattn
from oracle import plan as oplan

from parity import TOL_BF16_REL, TOL_LSE_ABS, rel_err

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _f64(t):
    """device bf16 / fp32 tensor -> float64 numpy"""
    import torch
    return t.detach().to(torch.float64).cpu().numpy()


def _run_both(ra):
    """plain entry points, then the direct ones on poisoned buffers; returns {family: (O, LSE, dQ, dK, dV)} as
    device tensors (clones)"""
    import torch
    import paper_2602_21788_amd as fcp
    out = {}
    ra.forward()
    ra.backward()
    torch.cuda.synchronize()
    assert fcp.fcp_scratch_status(ra.scratch_f)[1] == 0 and fcp.fcp_scratch_status(ra.scratch_b)[1] == 0
    out["plain"] = [t.clone() for t in (ra.o, ra.lse, ra.dq, ra.dk, ra.dv)]
    for t in (ra.o, ra.lse, ra.o_part, ra.lse_part, ra.dq_acc, ra.dk_acc, ra.dv_acc, ra.dq, ra.dk, ra.dv):
        t.fill_(float("nan"))
    ra.forward_direct()
    ra.backward_direct()
    torch.cuda.synchronize()
    assert fcp.fcp_scratch_status(ra.scratch_f)[1] == 0 and fcp.fcp_scratch_status(ra.scratch_b)[1] == 0
    out["direct"] = [t.clone() for t in (ra.o, ra.lse, ra.dq, ra.dk, ra.dv)]
    for fam in out:
        for name, t in zip(("O", "LSE", "dQ", "dK", "dV"), out[fam]):
            assert bool(torch.isfinite(t.float()).all()), (fam, name)
    return out


def full_size_sampled(cfg, kv_heads, stride, tail_keys=300):
    """cfg: index into the five workloads, or a Workload"""
    import torch
    from paper_2602_21788_amd.rank import RankAttention
    wl = cfg if isinstance(cfg, synth.Workload) else synth.make_workload(cfg)
    q, k, v, do = synth.draw_qkvdo(wl)
    cu = wl.cu_seqlens
    G = wl.hq // wl.hkv
    ra = RankAttention(wl.seq_lens, wl.cp_degree, wl.rank, wl.hq, wl.hkv, wl.head_dim, wl.softmax_scale)
    ochunks, owork = oplan.shard_plan(wl.seq_lens, wl.cp_degree)
    assert ra.chunks.tobytes() == ochunks.tobytes() and ra.work_all.tobytes() == owork.tobytes()
    rows = oplan.rank_rows(ochunks, cu, wl.rank)
    assert len(rows) == ra.tq
    sel = np.arange(0, len(rows), stride)
    _say(f"{wl.name} rank {wl.rank}: {ra.tq} rows, {ra.n_work} work items, {ra.n_parts} partial slots; "
         f"{len(sel)} sampled rows (every {stride}th), KV heads {kv_heads}")

    # ---- dense run --------------------------------------------------------------------------------------------
    ra.set_inputs(q, k, v, do)
    dense = _run_both(ra)
    # the tails of the rank's last and of its longest chunk: keys that only the chunk's rows after them see
    # (candidates: per sequence, the rank's last chunk of it)
    live = {}
    for c in ra.my_chunks:
        if c["len"] > 0:
            live[int(c["seq"])] = c
    live = list(live.values())
    picks = {int(cu[c["seq"]]) + int(c["seq_start"]) + int(c["len"]): int(c["len"])
             for c in (max(live, key=lambda c: int(cu[c["seq"]]) + int(c["seq_start"])), max(live, key=lambda c: int(c["len"])))}
    tails = []
    for chunk_end, clen in sorted(picks.items()):
        tk = np.arange(chunk_end - min(tail_keys, clen), chunk_end, dtype=np.int64)
        tr = rows[(rows >= tk[0]) & (rows < chunk_end)]
        later = rows[rows >= chunk_end]          # no later row of the rank may belong to the same sequence
        seq = int(np.searchsorted(cu, tk[0], side="right") - 1)
        assert not ((later >= cu[seq]) & (later < cu[seq + 1])).any()
        tails.append((tk, tr))
    refs = {}
    for kvh in kv_heads:
        hs = slice(kvh * G, (kvh + 1) * G)
        qs, dos = np.ascontiguousarray(q[:, hs]), np.ascontiguousarray(do[:, hs])
        ks, vs = np.ascontiguousarray(k[:, kvh:kvh + 1]), np.ascontiguousarray(v[:, kvh:kvh + 1])
        O_ref, LSE_ref = oattn.attn_fwd(qs, ks, vs, cu, wl.softmax_scale, rows[sel])
        dQ_ref = oattn.attn_dq(qs, ks, vs, dos, cu, wl.softmax_scale, rows[sel], O_ref, LSE_ref)
        tail_refs = []
        for tk, tr in tails:
            O_t, LSE_t = oattn.attn_fwd(qs, ks, vs, cu, wl.softmax_scale, tr)
            tail_refs.append(oattn.attn_dkv(qs, ks, vs, dos, cu, wl.softmax_scale, tr, O_t, LSE_t, keys=tk))
        refs[kvh] = (qs, ks, vs, O_ref, LSE_ref)
        do_sum = synth.bf16_bits_to_f64(dos[rows]).sum(axis=(0, 1))        # [D]: all rank rows, the group's heads
        for fam, (O, LSE, dQ, dK, dV) in dense.items():
            e = {"O": rel_err(_f64(O[sel][:, hs]), O_ref),
                 "LSE": float(np.abs(_f64(LSE[hs][:, sel]).T - LSE_ref).max()),
                 "dQ": rel_err(_f64(dQ[sel][:, hs]), dQ_ref),
                 "dK_tail": max(rel_err(_f64(dK[tk[0]:tk[-1] + 1, kvh:kvh + 1]), r[0]) for (tk, _), r in zip(tails, tail_refs)),
                 "dV_tail": max(rel_err(_f64(dV[tk[0]:tk[-1] + 1, kvh:kvh + 1]), r[1]) for (tk, _), r in zip(tails, tail_refs))}
            dv_all, dk_all = _f64(dV[:, kvh]), _f64(dK[:, kvh])
            # identities over all keys; the bf16 rounding of ~tkv summands of size <= max|dV| adds up like a random walk
            noise = 2.0 ** -8 * np.sqrt(dv_all.shape[0])
            e["sum_dV"] = float(np.abs(dv_all.sum(axis=0) - do_sum).max() / max(np.abs(do_sum).max(), noise * np.abs(dv_all).max()))
            e["sum_dK"] = float(np.abs(dk_all.sum(axis=0)).max() / (noise * np.abs(dk_all).max()))
            _say(f"  dense  {fam:6s} kv head {kvh}: " + ", ".join(f"{a} {b:.2e}" for a, b in e.items()))
            assert e["LSE"] <= TOL_LSE_ABS, (fam, kvh, e)
            for name in ("O", "dQ", "dK_tail", "dV_tail"):
                assert e[name] <= TOL_BF16_REL, (fam, kvh, name, e)
            assert e["sum_dV"] <= TOL_BF16_REL and e["sum_dK"] <= 4.0, (fam, kvh, e)
    del dense

    # ---- sparse run: dO lives on the sampled rows only ------------------------------------------------------------
    do_sp = np.zeros_like(do)
    do_sp[rows[sel]] = do[rows[sel]]
    ra.set_inputs(q, k, v, do_sp)
    sparse = _run_both(ra)
    for kvh in kv_heads:
        hs = slice(kvh * G, (kvh + 1) * G)
        qs, ks, vs, O_ref, LSE_ref = refs[kvh]
        dos = np.ascontiguousarray(do_sp[:, hs])
        dQ_ref = oattn.attn_dq(qs, ks, vs, dos, cu, wl.softmax_scale, rows[sel], O_ref, LSE_ref)
        dK_ref, dV_ref = oattn.attn_dkv(qs, ks, vs, dos, cu, wl.softmax_scale, rows[sel], O_ref, LSE_ref)
        unsel = np.ones(len(rows), bool)
        unsel[sel] = False
        for fam, (O, LSE, dQ, dK, dV) in sparse.items():
            e = {"dQ": rel_err(_f64(dQ[sel][:, hs]), dQ_ref),
                 "dK": rel_err(_f64(dK[:, kvh:kvh + 1]), dK_ref),
                 "dV": rel_err(_f64(dV[:, kvh:kvh + 1]), dV_ref)}
            _say(f"  sparse {fam:6s} kv head {kvh}: " + ", ".join(f"{a} {b:.2e}" for a, b in e.items()))
            for name in e:
                assert e[name] <= TOL_BF16_REL, (fam, kvh, name, e)
            # rows without an upstream gradient get none
            assert float(dQ[torch.from_numpy(np.nonzero(unsel)[0]).to(dQ.device)][:, hs].float().abs().max()) == 0.0, fam


def test_cfg3_L131072_degree5_rank2_full_size_sampled():
    """One 131072-token sequence at CP degree 5, rank 2 (chunks 2 and 7, 26214 rows, five partial slots)."""
    full_size_sampled(3, kv_heads=(3,), stride=29)


def test_cfg4_multimodal_imbalance_rank0_full_size_sampled():
    """49152 tokens at degree 6 plus 64 short sequences, 40 query / 8 KV heads (five query heads per KV head: the
    256-row forward units), rank 0: a zigzag pair of the long sequence and all the short ones."""
    full_size_sampled(4, kv_heads=(6,), stride=23)


def test_cfg2_packed32k_rank0_full_size_both_families_against_the_oracle():
    """The benchmark workload: the direct entry points (what bench.py times) and the plain ones, each against the
    oracle on sampled rows, the tail keys and - through the sparse-dO run - every key of one KV head."""
    full_size_sampled(2, kv_heads=(2,), stride=31)


def test_one_131072_token_sequence_unsharded_32_heads_largest_rank_the_backward_accepts():
    """131072 rows x 32 heads x 128 on one rank (2^29 elements per tensor, 1 GiB of bf16 each: the bf16 rows of the one
    work item span 2^30 bytes, the largest 32-bit offsets the kernels form; 2 GiB fp32 accumulators and partial O), one
    1024-tile work item per list."""
    wl = synth.custom_workload([131072], [1], 32, 8, 128, rank=0, seed=11, name="L131072_d1_h32x8_D128")
    full_size_sampled(wl, kv_heads=(5,), stride=997, tail_keys=200)
