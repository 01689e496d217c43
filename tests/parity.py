"""Helpers of the GPU parity tests: run one rank on the GPU through the C ABI and the
oracle on the CPU for the same seeded inputs, and compare to the stated tolerances.

Tolerances (the build's target statement): max|x_gpu - x_ref| / max|x_ref| <= 2e-2 for the
bf16 tensors O, dQ, dK, dV; max|LSE_gpu - LSE_ref| <= 1e-3 (absolute) for fp32 LSE.
"""
import numpy as np

import fcp_synth as synth
from oracle import attn as oattn
from oracle import plan as oplan

TOL_BF16_REL = 2e-2
TOL_LSE_ABS = 1e-3


def rel_err(got, ref):
    ref = np.asarray(ref, np.float64)
    got = np.asarray(got, np.float64)
    denom = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (denom if denom > 0 else 1.0))


def bf16_tensor_to_f64(t):
    import torch
    return synth.bf16_bits_to_f64(t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16))


def check_rank(wl, q, k, v, do, rank, backward=True, check_partials=False, label="", spans=None, base_rank=None,
               direct=True):
    """Full element-by-element comparison of one rank (small workloads).  spans: full-attention spans
    [(seq, start, len), ...] of a mixed mask, None = causal.  direct=False: the work list is longer than the direct
    entry points take; they must refuse it, and only the plain ones are compared."""
    import torch
    from paper_2602_21788_amd.rank import RankAttention
    ra = RankAttention(wl.seq_lens, wl.cp_degree, rank, wl.hq, wl.hkv, wl.head_dim, wl.softmax_scale, spans=spans,
                       base_rank=base_rank)
    ochunks, owork = oplan.shard_plan(wl.seq_lens, wl.cp_degree, base_rank, spans=spans)
    sid = None if spans is None else oplan.span_ids(wl.seq_lens, spans)
    assert ra.chunks.tobytes() == ochunks.tobytes() and ra.work_all.tobytes() == owork.tobytes()
    rows = oplan.rank_rows(ochunks, wl.cu_seqlens, rank)
    if len(rows) == 0:
        return None
    ra.set_inputs(q, k, v, do if backward else None)
    ra.forward()
    torch.cuda.synchronize()
    n_tiles, n_rej = __import__("paper_2602_21788_amd").fcp_scratch_status(ra.scratch_f)
    assert n_rej == 0, f"{label}: {n_rej} work items rejected"
    O_ref, LSE_ref = oattn.attn_fwd(q, k, v, wl.cu_seqlens, wl.softmax_scale, rows, span_id=sid)
    O = bf16_tensor_to_f64(ra.o)
    LSE = ra.lse.cpu().numpy().astype(np.float64).T          # [tq, hq]
    res = {"O": rel_err(O, O_ref), "LSE": float(np.abs(LSE - LSE_ref).max())}
    assert np.isfinite(O).all() and np.isfinite(LSE).all(), label
    assert res["O"] <= TOL_BF16_REL, (label, res)
    assert res["LSE"] <= TOL_LSE_ABS, (label, res)
    # The direct forward (rows fed by one work item written once by the kernel, the others merged) on poisoned
    # buffers: the same bar, and the same values as partial results + merge up to the bf16 rounding of O.
    if not direct:
        return _plain_only(ra, wl, q, k, v, do, rows, O_ref, LSE_ref, sid, backward, res, label)
    for t in (ra.o, ra.lse, ra.o_part, ra.lse_part):
        t.fill_(float("nan"))
    ra.forward_direct()
    torch.cuda.synchronize()
    assert __import__("paper_2602_21788_amd").fcp_scratch_status(ra.scratch_f)[1] == 0, label
    O_d = bf16_tensor_to_f64(ra.o)
    LSE_d = ra.lse.cpu().numpy().astype(np.float64).T
    assert np.isfinite(O_d).all() and not np.isnan(LSE_d).any(), (label, "direct forward")
    res["O_direct"] = rel_err(O_d, O_ref)
    res["LSE_direct"] = float(np.abs(LSE_d - LSE_ref).max())
    assert res["O_direct"] <= TOL_BF16_REL and res["LSE_direct"] <= TOL_LSE_ABS, (label, "direct forward", res)
    assert rel_err(O_d, O) <= 2.0 ** -7 and np.abs(LSE_d - LSE).max() <= 1e-5, (label, "direct vs partial + merge")
    ra.forward()                      # (the partial results are looked at below)
    torch.cuda.synchronize()
    if check_partials:
        qf, kf, vf = (synth.bf16_bits_to_f64(x) for x in (q, k, v))
        Op_ref, Lp_ref = oplan.rank_partials(qf, kf, vf, wl.cu_seqlens, ochunks, owork, rank, wl.softmax_scale, span_id=sid)
        Op = ra.o_part.cpu().numpy().astype(np.float64)
        Lp = ra.lse_part.cpu().numpy().astype(np.float64).transpose(0, 2, 1)
        assert Op.shape == Op_ref.shape
        fin = np.isfinite(Lp_ref)
        assert (np.isneginf(Lp) == ~fin).all(), label          # uncovered rows are -inf, exactly those
        assert np.abs(Lp[fin] - Lp_ref[fin]).max() <= TOL_LSE_ABS, label
        err = np.abs(np.where(fin[..., None], Op - Op_ref, 0.0)).max() / np.abs(Op_ref).max()
        assert err <= TOL_BF16_REL, (label, err)
        res["O_part"] = float(err)
    if backward:
        ra.backward()
        torch.cuda.synchronize()
        n_tiles, n_rej = __import__("paper_2602_21788_amd").fcp_scratch_status(ra.scratch_b)
        assert n_rej == 0, f"{label}: {n_rej} work items rejected (bwd)"
        dQ_ref = oattn.attn_dq(q, k, v, do, wl.cu_seqlens, wl.softmax_scale, rows, O_ref, LSE_ref, span_id=sid)
        dK_ref, dV_ref = oattn.attn_dkv(q, k, v, do, wl.cu_seqlens, wl.softmax_scale, rows, O_ref, LSE_ref, span_id=sid)
        got = {"dQ": bf16_tensor_to_f64(ra.dq), "dK": bf16_tensor_to_f64(ra.dk), "dV": bf16_tensor_to_f64(ra.dv)}
        for name, ref in (("dQ", dQ_ref), ("dK", dK_ref), ("dV", dV_ref)):
            assert np.isfinite(got[name]).all(), (label, name)
            res[name] = rel_err(got[name], ref)
            assert res[name] <= TOL_BF16_REL, (label, name, res)
        res["_dK_acc"] = ra.dk_acc.cpu().numpy().astype(np.float64)
        res["_dV_acc"] = ra.dv_acc.cpu().numpy().astype(np.float64)
        # The direct backward (rows owned by one unit written as bf16 by their kernel) on poisoned buffers: it must
        # neither need cleared accumulators nor leave any output row unwritten, and meets the same bar.
        for t in (ra.dq_acc, ra.dk_acc, ra.dv_acc, ra.dq, ra.dk, ra.dv):
            t.fill_(float("nan"))
        ra.backward_direct()
        torch.cuda.synchronize()
        n_tiles, n_rej = __import__("paper_2602_21788_amd").fcp_scratch_status(ra.scratch_b)
        assert n_rej == 0, f"{label}: {n_rej} work items rejected (direct bwd)"
        direct = {"dQ": bf16_tensor_to_f64(ra.dq), "dK": bf16_tensor_to_f64(ra.dk), "dV": bf16_tensor_to_f64(ra.dv)}
        for name, ref in (("dQ", dQ_ref), ("dK", dK_ref), ("dV", dV_ref)):
            assert np.isfinite(direct[name]).all(), (label, name, "direct")
            res[name + "_direct"] = rel_err(direct[name], ref)
            assert res[name + "_direct"] <= TOL_BF16_REL, (label, name, "direct", res)
            # against the accumulating path: the same arithmetic, except for the order of the fp32 atomics
            assert rel_err(direct[name], got[name]) <= 2.0 ** -7, (label, name, "direct vs accumulating")
    return res


def _plain_only(ra, wl, q, k, v, do, rows, O_ref, LSE_ref, sid, backward, res, label):
    """Work lists beyond the direct entry points' limit: those refuse the list (and launch nothing), the plain
    backward is compared with the oracle."""
    import torch
    import pytest
    from paper_2602_21788_amd.binding import FcpError, FCP_ERR_UNSUPPORTED
    with pytest.raises(FcpError) as ei:
        ra.forward_steps_direct()
    assert ei.value.code == FCP_ERR_UNSUPPORTED, label
    if backward:
        with pytest.raises(FcpError) as ei:
            ra.backward_steps_direct()
        assert ei.value.code == FCP_ERR_UNSUPPORTED, label
        ra.backward()
        torch.cuda.synchronize()
        assert __import__("paper_2602_21788_amd").fcp_scratch_status(ra.scratch_b)[1] == 0, label
        dQ_ref = oattn.attn_dq(q, k, v, do, wl.cu_seqlens, wl.softmax_scale, rows, O_ref, LSE_ref, span_id=sid)
        dK_ref, dV_ref = oattn.attn_dkv(q, k, v, do, wl.cu_seqlens, wl.softmax_scale, rows, O_ref, LSE_ref, span_id=sid)
        for name, t, ref in (("dQ", ra.dq, dQ_ref), ("dK", ra.dk, dK_ref), ("dV", ra.dv, dV_ref)):
            got = bf16_tensor_to_f64(t)
            assert np.isfinite(got).all(), (label, name)
            res[name] = rel_err(got, ref)
            assert res[name] <= TOL_BF16_REL, (label, name, res)
    return res
