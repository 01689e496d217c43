"""fcp_attn_fwd_step_static (the entry point that allocates nothing: its work area is a static device array inside the
library) against fcp_attn_fwd_step with a caller-owned scratch buffer, through the C ABI: two calls in a row on the
same GPU, the second with a smaller input, so that whatever the first call left in the shared area is there when the
second one runs.  Same kernels and the same tile records, so the partial results must be identical; they are also held
to the oracle's bar (LSE 1e-3 absolute, O 2e-2 of max|ref|) after the merge."""
import numpy as np
import pytest

import fcp_synth as synth
from oracle import attn as oattn
from oracle import plan as oplan

from parity import TOL_BF16_REL, TOL_LSE_ABS, bf16_tensor_to_f64, rel_err

pytestmark = pytest.mark.gpu


def _case(lens, deg, rank, hq, hkv, D, seed):
    import torch
    import paper_2602_21788_amd as fcp
    from paper_2602_21788_amd.rank import RankAttention
    wl = synth.custom_workload(lens, deg, hq=hq, hkv=hkv, head_dim=D, rank=rank, seed=seed)
    q, k, v, _ = synth.draw_qkvdo(wl)
    ra = RankAttention(wl.seq_lens, wl.cp_degree, rank, hq, hkv, D, wl.softmax_scale)
    ra.set_inputs(q, k, v, None)
    print(f"static work area: lens {list(lens)} degrees {list(deg)} rank {rank}: {ra.tq} rows, {ra.n_work} items", flush=True)
    # existing entry point, caller-owned scratch
    ra.o_part.fill_(float("nan")); ra.lse_part.fill_(float("nan"))
    ra.forward_steps()
    torch.cuda.synchronize()
    want_o, want_l = ra.o_part.clone(), ra.lse_part.clone()
    # the static one, on poisoned outputs
    ra.o_part.fill_(float("nan")); ra.lse_part.fill_(float("nan"))
    fcp.fcp_attn_fwd_step_static(ra.q, ra.k, ra.v, ra.cu_d, ra.work_d, ra.n_parts, ra.scale, ra.o_part, ra.lse_part)
    torch.cuda.synchronize()
    assert not torch.isnan(ra.lse_part).any()
    assert torch.equal(ra.lse_part, want_l)
    covered = torch.isfinite(want_l).transpose(1, 2).unsqueeze(-1).expand_as(want_o)      # [parts, tq, hq, D]
    assert torch.equal(torch.where(covered, ra.o_part, torch.zeros_like(ra.o_part)),
                       torch.where(covered, want_o, torch.zeros_like(want_o)))
    # and against the oracle, after the merge
    ra.merge()
    torch.cuda.synchronize()
    chunks, _ = oplan.shard_plan(wl.seq_lens, wl.cp_degree)
    rows = oplan.rank_rows(chunks, wl.cu_seqlens, rank)
    O_ref, LSE_ref = oattn.attn_fwd(q, k, v, wl.cu_seqlens, wl.softmax_scale, rows)
    assert rel_err(bf16_tensor_to_f64(ra.o), O_ref) <= TOL_BF16_REL
    assert np.abs(ra.lse.cpu().numpy().astype(np.float64).T - LSE_ref).max() <= TOL_LSE_ABS


def test_static_work_area_two_calls_second_smaller():
    _case([1500, 130, 700, 64, 333], [3, 1, 2, 1, 1], rank=0, hq=8, hkv=2, D=128, seed=201)
    _case([257, 40], [2, 1], rank=1, hq=8, hkv=2, D=128, seed=202)


def test_static_work_area_rejects_what_does_not_fit():
    """A call whose tile list cannot fit the static area is refused with a capacity error before anything is launched."""
    import ctypes
    import torch
    from paper_2602_21788_amd import binding as B
    need = B.fcp_scratch_bytes(B.FCP_SCRATCH_FWD, 1 << 22, 1 << 22, 8, 8, 128, 100000, 4)
    assert need > 2 * 1024 * 1024
    t = torch.zeros(64, dtype=torch.float32, device="cuda")
    p = ctypes.c_void_p(t.data_ptr())
    rc = B.lib().fcp_attn_fwd_step_static(p, p, p, p, 1, p, 100000, 4, 1 << 22, 1 << 22, 8, 8, 128, 0.1, p, p, None)
    assert rc == B.FCP_ERR_CAPACITY and b"static" in B.lib().fcp_last_error()
