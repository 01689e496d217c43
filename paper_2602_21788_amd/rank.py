"""One CP rank's attention pass wired from the C-ABI calls (used by tests, bench and smoke).

Only buffer management lives here: gather the rank's query rows named by the chunk table,
allocate device tensors with torch, and call the library in the order
  fcp_attn_fwd_step (all ring steps in one launch) -> fcp_lse_merge
  fcp_attn_bwd_delta -> fcp_attn_bwd_step -> fcp_grad_finalize (dQ, dK, dV).
All KV chunks of the rank's groups are resident in one pool, as if every ring step's
block had already arrived.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def _bits_to_dev(bits: np.ndarray, device) -> torch.Tensor:
    """uint16 bf16 bit patterns -> torch.bfloat16 device tensor (no value change)."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.to(device).view(torch.bfloat16)


def dev_to_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


class RankAttention:
    """Buffers and launches for one rank of a planned batch."""

    def __init__(self, seq_lens, cp_degree, rank, hq, hkv, head_dim, softmax_scale=None,
                 base_rank=None, device="cuda:0", spans=None):
        """spans: optional full-attention spans [(seq, start, len), ...] (mixed mask); None = causal."""
        self.device = torch.device(device)
        self.hq, self.hkv, self.D = hq, hkv, head_dim
        self.scale = float(softmax_scale) if softmax_scale is not None else 1.0 / float(np.sqrt(head_dim))
        self.seq_lens = np.asarray(seq_lens, np.int32)
        self.spans = spans
        if spans is None:
            self.chunks, self.work_all = B.fcp_shard_plan(seq_lens, cp_degree, base_rank)
        else:
            self.chunks, self.work_all = B.fcp_shard_plan_mixed(seq_lens, cp_degree, spans, base_rank)
        self.rank = rank
        self.my_chunks = self.chunks[self.chunks["rank"] == rank]
        self.work = np.ascontiguousarray(self.work_all[self.work_all["rank"] == rank])
        cu = np.zeros(len(self.seq_lens) + 1, np.int32)
        np.cumsum(self.seq_lens, out=cu[1:])
        self.cu = cu
        self.tkv = int(cu[-1])
        self.tq = int(self.my_chunks["len"].sum())
        self.n_parts = int(self.work["step"].max()) + 1 if len(self.work) else 1
        rows = [np.arange(int(cu[c["seq"]]) + int(c["seq_start"]), int(cu[c["seq"]]) + int(c["seq_start"]) + int(c["len"]),
                          dtype=np.int64) for c in self.my_chunks]
        self.rows = np.concatenate(rows) if rows else np.zeros(0, np.int64)
        dev = self.device
        self.cu_d = torch.from_numpy(cu).to(dev)
        self.work_d = torch.from_numpy(self.work.view(np.uint8).copy()).to(dev) if len(self.work) else \
            torch.zeros(B.WORK_DTYPE.itemsize, dtype=torch.uint8, device=dev)[:0]
        self.n_work = len(self.work)
        self.q_limit_d = self.k_from_d = None
        if spans is not None:
            self.q_limit, self.k_from, self.eta = B.fcp_mask_tables(self.seq_lens, spans, self.chunks, rank)
            self.q_limit_d = torch.from_numpy(self.q_limit).to(dev)
            self.k_from_d = torch.from_numpy(self.k_from).to(dev)
        nb_f = B.fcp_scratch_bytes(B.FCP_SCRATCH_FWD, self.tq, self.tkv, hq, hkv, head_dim, self.n_work, self.n_parts)
        nb_b = B.fcp_scratch_bytes(B.FCP_SCRATCH_BWD, self.tq, self.tkv, hq, hkv, head_dim, self.n_work, self.n_parts)
        self.scratch_f = torch.empty(nb_f, dtype=torch.uint8, device=dev)
        self.scratch_b = torch.empty(nb_b, dtype=torch.uint8, device=dev)
        self.q = self.k = self.v = self.d_o = None

    # -- inputs ---------------------------------------------------------------------
    def set_inputs(self, q_bits, k_bits, v_bits, do_bits=None):
        """Unsharded bf16 bit tensors [T,H,D]; the rank's query rows are gathered here."""
        self.q = _bits_to_dev(np.ascontiguousarray(q_bits[self.rows]), self.device)
        self.k = _bits_to_dev(k_bits, self.device)
        self.v = _bits_to_dev(v_bits, self.device)
        self.d_o = None if do_bits is None else _bits_to_dev(np.ascontiguousarray(do_bits[self.rows]), self.device)
        self._alloc_outputs()

    def set_random_inputs(self, seed=0):
        """Device-side N(0,1) bf16 inputs (benchmark use; values differ from the numpy generator)."""
        g = torch.Generator(device=self.device).manual_seed(seed)
        mk = lambda *s: torch.randn(*s, generator=g, device=self.device, dtype=torch.float32).to(torch.bfloat16)
        self.q, self.d_o = mk(self.tq, self.hq, self.D), mk(self.tq, self.hq, self.D)
        self.k, self.v = mk(self.tkv, self.hkv, self.D), mk(self.tkv, self.hkv, self.D)
        self._alloc_outputs()

    def _alloc_outputs(self):
        dev, tq, hq, hkv, D = self.device, self.tq, self.hq, self.hkv, self.D
        self.o_part = torch.empty(self.n_parts, tq, hq, D, dtype=torch.float32, device=dev)
        self.lse_part = torch.empty(self.n_parts, hq, tq, dtype=torch.float32, device=dev)
        self.o = torch.empty(tq, hq, D, dtype=torch.bfloat16, device=dev)
        self.lse = torch.empty(hq, tq, dtype=torch.float32, device=dev)
        self.delta = torch.empty(hq, tq, dtype=torch.float32, device=dev)
        self.dq_acc = torch.empty(tq, hq, D, dtype=torch.float32, device=dev)
        self.dk_acc = torch.empty(self.tkv, hkv, D, dtype=torch.float32, device=dev)
        self.dv_acc = torch.empty(self.tkv, hkv, D, dtype=torch.float32, device=dev)
        self.dq = torch.empty(tq, hq, D, dtype=torch.bfloat16, device=dev)
        self.dk = torch.empty(self.tkv, hkv, D, dtype=torch.bfloat16, device=dev)
        self.dv = torch.empty(self.tkv, hkv, D, dtype=torch.bfloat16, device=dev)

    # -- passes -----------------------------------------------------------------------
    def forward_steps(self, stream=None):
        if self.spans is not None:
            B.fcp_attn_fwd_step_mixed(self.q, self.k, self.v, self.cu_d, self.work_d, self.n_parts, self.scale,
                                      self.q_limit_d, self.o_part, self.lse_part, self.scratch_f, stream)
            return
        B.fcp_attn_fwd_step(self.q, self.k, self.v, self.cu_d, self.work_d, self.n_parts, self.scale,
                            self.o_part, self.lse_part, self.scratch_f, stream)

    def forward_running(self, stream=None):
        """The forward pass as one fcp_attn_fwd_step_running call per ring step (no partials, no merge): the
        results land in self.o (bf16), self.lse and self.o_run (fp32)."""
        if not hasattr(self, "step_work_d"):
            self.step_work_d = []
            for s in range(self.n_parts):
                w = np.ascontiguousarray(self.work[self.work["step"] == s])
                if len(w):
                    self.step_work_d.append(torch.from_numpy(w.view(np.uint8).copy()).to(self.device))
            self.o_run = torch.empty(self.tq, self.hq, self.D, dtype=torch.float32, device=self.device)
        self.lse.fill_(float("-inf"))
        for w in self.step_work_d:
            B.fcp_attn_fwd_step_running(self.q, self.k, self.v, self.cu_d, w, self.scale, self.o_run, self.lse,
                                        self.scratch_f, o_out=self.o, q_limit=self.q_limit_d, stream=stream)

    def merge(self, stream=None):
        B.fcp_lse_merge(self.o_part, self.lse_part, self.o, self.lse, stream)

    def forward(self, stream=None):
        self.forward_steps(stream)
        self.merge(stream)

    # The same results with the rows that one work item feeds written once, as bf16, by the forward kernel.
    def forward_steps_direct(self, stream=None):
        B.fcp_attn_fwd_step_direct(self.q, self.k, self.v, self.cu_d, self.work_d, self.n_parts, self.scale, self.o_part,
                                   self.lse_part, self.o, self.lse, self.scratch_f,
                                   q_limit=self.q_limit_d if self.spans is not None else None, stream=stream)

    def merge_direct(self, stream=None):
        B.fcp_lse_merge_direct(self.o_part, self.lse_part, self.o, self.lse, self.tkv, self.scratch_f, self.n_work, stream)

    def forward_direct(self, stream=None):
        self.forward_steps_direct(stream)
        self.merge_direct(stream)

    def zero_grads(self):
        self.dq_acc.zero_(); self.dk_acc.zero_(); self.dv_acc.zero_()

    def backward_delta(self, stream=None):
        B.fcp_attn_bwd_delta(self.o, self.d_o, self.delta, stream)

    def backward_steps(self, stream=None):
        if self.spans is not None:
            B.fcp_attn_bwd_step_mixed(self.q, self.k, self.v, self.d_o, self.lse, self.delta, self.cu_d, self.work_d,
                                      self.scale, self.q_limit_d, self.k_from_d, self.dq_acc, self.dk_acc, self.dv_acc,
                                      self.scratch_b, stream)
            return
        B.fcp_attn_bwd_step(self.q, self.k, self.v, self.d_o, self.lse, self.delta, self.cu_d, self.work_d,
                            self.scale, self.dq_acc, self.dk_acc, self.dv_acc, self.scratch_b, stream)

    def finalize(self, stream=None):
        B.fcp_grad_finalize(self.dq_acc, self.dq, stream)
        B.fcp_grad_finalize(self.dk_acc, self.dk, stream)
        B.fcp_grad_finalize(self.dv_acc, self.dv, stream)

    def backward(self, stream=None):
        self.zero_grads()
        self.backward_delta(stream)
        self.backward_steps(stream)
        self.finalize(stream)

    # The same results without clearing and converting every accumulator row: rows owned by one unit of work are
    # written as bf16 by the kernel that computes them (fcp_attn_bwd_step_direct + fcp_grad_finalize_direct).
    def backward_steps_direct(self, stream=None):
        B.fcp_attn_bwd_step_direct(self.q, self.k, self.v, self.d_o, self.lse, self.delta, self.cu_d, self.work_d,
                                   self.scale, self.dq_acc, self.dk_acc, self.dv_acc, self.dq, self.dk, self.dv,
                                   self.scratch_b, q_limit=self.q_limit_d if self.spans is not None else None,
                                   k_from=self.k_from_d if self.spans is not None else None, stream=stream)

    def finalize_direct(self, stream=None):
        B.fcp_grad_finalize_direct(self.dq_acc, self.dk_acc, self.dv_acc, self.dq, self.dk, self.dv, self.scratch_b,
                                   self.n_work, stream)

    def backward_direct(self, stream=None):
        self.backward_delta(stream)
        self.backward_steps_direct(stream)
        self.finalize_direct(stream)
