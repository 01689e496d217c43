"""Thin ctypes binding of libfcp.so: the same entry points as include/fcp.h, argument
marshalling only.  Device buffers are torch tensors (PyTorch is used for device memory and
streams, nothing else); every step of the path runs in the library's own kernels.

There is no fallback: if libfcp.so is missing or does not load, importing a function from
here raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libfcp.so")

FCP_OK, FCP_ERR_INVALID_ARG, FCP_ERR_CAPACITY, FCP_ERR_UNSUPPORTED, FCP_ERR_HIP = 0, -1, -2, -3, -4
FCP_SCRATCH_FWD, FCP_SCRATCH_BWD = 0, 1

CHUNK_DTYPE = np.dtype([("seq", "<i4"), ("rank", "<i4"), ("chunk", "<i4"),
                        ("seq_start", "<i4"), ("len", "<i4"), ("local_off", "<i4")])
WORK_DTYPE = np.dtype([("seq", "<i4"), ("rank", "<i4"), ("step", "<i4"),
                       ("q_local_off", "<i4"), ("q_seq_start", "<i4"), ("q_len", "<i4"),
                       ("n_seg", "<i4"), ("k_seq_start", "<i4", (2,)), ("k_len", "<i4", (2,))])
SPAN_DTYPE = np.dtype([("seq", "<i4"), ("start", "<i4"), ("len", "<i4")])

EXPORTS = ["fcp_last_error", "fcp_shard_plan", "fcp_plan_groups", "fcp_scratch_bytes", "fcp_attn_fwd_step", "fcp_lse_merge",
           "fcp_attn_bwd_delta", "fcp_attn_bwd_step", "fcp_grad_finalize", "fcp_scratch_status",
           "fcp_group_shard_args", "fcp_attn_fwd_step_running", "fcp_shard_plan_mixed", "fcp_mask_tables", "fcp_attn_fwd_step_mixed", "fcp_attn_bwd_step_mixed",
           "fcp_attn_bwd_step_direct", "fcp_grad_finalize_direct", "fcp_attn_fwd_step_direct", "fcp_lse_merge_direct", "fcp_attn_fwd_step_static"]


class FcpError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libfcp error {code}: {msg}")
        self.code = code


_lib = None


def lib() -> ctypes.CDLL:
    """Loads libfcp.so (built in-tree by paper_2602_21788_amd.build); builds it if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            from . import build as _build
            _build.build()
        # torch first: it ships its own HIP runtime, and a process must not end up with two (libfcp.so loaded before
        # torch would bind to the system's copy, and the second runtime to start finds no device)
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        P, I32, I64, F, SZ = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
        L.fcp_last_error.restype = ctypes.c_char_p
        L.fcp_last_error.argtypes = []
        L.fcp_shard_plan.restype = ctypes.c_int
        L.fcp_shard_plan.argtypes = [P, P, P, I32, P, I64, P, P, I64, P]
        L.fcp_plan_groups.restype = ctypes.c_int
        L.fcp_plan_groups.argtypes = [P, P, I32, I32, I64, P, P, P, P, P, P, P]
        L.fcp_scratch_bytes.restype = SZ
        L.fcp_scratch_bytes.argtypes = [ctypes.c_int, I32, I32, I32, I32, I32, I64, I32]
        L.fcp_attn_fwd_step.restype = ctypes.c_int
        L.fcp_attn_fwd_step.argtypes = [P, P, P, P, I32, P, I64, I32, I32, I32, I32, I32, I32, F, P, P, P, SZ, P]
        L.fcp_attn_fwd_step_static.restype = ctypes.c_int
        L.fcp_attn_fwd_step_static.argtypes = [P, P, P, P, I32, P, I64, I32, I32, I32, I32, I32, I32, F, P, P, P]
        L.fcp_lse_merge.restype = ctypes.c_int
        L.fcp_lse_merge.argtypes = [P, P, I32, I32, I32, I32, P, P, P]
        L.fcp_attn_bwd_delta.restype = ctypes.c_int
        L.fcp_attn_bwd_delta.argtypes = [P, P, I32, I32, I32, P, P]
        L.fcp_attn_bwd_step.restype = ctypes.c_int
        L.fcp_attn_bwd_step.argtypes = [P, P, P, P, P, P, P, I32, P, I64, I32, I32, I32, I32, I32, F, P, P, P, P, SZ, P]
        L.fcp_grad_finalize.restype = ctypes.c_int
        L.fcp_grad_finalize.argtypes = [P, P, I64, P]
        L.fcp_scratch_status.restype = ctypes.c_int
        L.fcp_scratch_status.argtypes = [P, P, P, P]
        L.fcp_group_shard_args.restype = ctypes.c_int
        L.fcp_group_shard_args.argtypes = [P, I32, P, P, I32, P, P]
        L.fcp_shard_plan_mixed.restype = ctypes.c_int
        L.fcp_shard_plan_mixed.argtypes = [P, P, P, I32, P, I32, P, I64, P, P, I64, P]
        L.fcp_mask_tables.restype = ctypes.c_int
        L.fcp_mask_tables.argtypes = [P, I32, P, I32, P, I64, I32, P, I64, P, P, P]
        L.fcp_attn_fwd_step_mixed.restype = ctypes.c_int
        L.fcp_attn_fwd_step_mixed.argtypes = [P, P, P, P, I32, P, I64, I32, I32, I32, I32, I32, I32, F, P, P, P, P, SZ, P]
        L.fcp_attn_fwd_step_running.restype = ctypes.c_int
        L.fcp_attn_fwd_step_running.argtypes = [P, P, P, P, I32, P, I64, I32, I32, I32, I32, I32, F, P, P, P, P, P, SZ, P]
        L.fcp_attn_bwd_step_mixed.restype = ctypes.c_int
        L.fcp_attn_bwd_step_mixed.argtypes = [P, P, P, P, P, P, P, I32, P, I64, I32, I32, I32, I32, I32, F, P, P, P, P, P, P,
                                              SZ, P]
        L.fcp_attn_bwd_step_direct.restype = ctypes.c_int
        L.fcp_attn_bwd_step_direct.argtypes = [P, P, P, P, P, P, P, I32, P, I64, I32, I32, I32, I32, I32, F, P, P, P, P, P, P,
                                               P, P, P, SZ, P]
        L.fcp_grad_finalize_direct.restype = ctypes.c_int
        L.fcp_grad_finalize_direct.argtypes = [P, P, P, P, P, P, P, I64, I32, I32, I32, I32, I32, P]
        L.fcp_attn_fwd_step_direct.restype = ctypes.c_int
        L.fcp_attn_fwd_step_direct.argtypes = [P, P, P, P, I32, P, I64, I32, I32, I32, I32, I32, I32, F, P, P, P, P, P, P, SZ, P]
        L.fcp_lse_merge_direct.restype = ctypes.c_int
        L.fcp_lse_merge_direct.argtypes = [P, P, I32, I32, I32, I32, I32, P, P, P, I64, P]
        _lib = L
    return _lib


def _check(rc: int):
    if rc != FCP_OK:
        raise FcpError(rc, lib().fcp_last_error().decode())


def _np_ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _dev_ptr(t):
    """Device pointer of a torch tensor (must be contiguous and on a GPU)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(int(getattr(stream, "cuda_stream", stream)))


# ---------------------------------------------------------------------------------------
def fcp_shard_plan(seq_lens, cp_degree, base_rank=None):
    """Host only.  Returns (chunks, work) numpy structured arrays (CHUNK_DTYPE, WORK_DTYPE)."""
    sl = np.ascontiguousarray(seq_lens, dtype=np.int32)
    cd = np.ascontiguousarray(cp_degree, dtype=np.int32)
    if sl.shape != cd.shape or sl.ndim != 1:
        raise ValueError("seq_lens and cp_degree must be 1-D and the same length")
    br = None if base_rank is None else np.ascontiguousarray(base_rank, dtype=np.int32)
    if br is not None and br.shape != sl.shape:
        raise ValueError("base_rank must match seq_lens")
    nc, nw = ctypes.c_int64(0), ctypes.c_int64(0)
    _check(lib().fcp_shard_plan(_np_ptr(sl), _np_ptr(cd), _np_ptr(br), len(sl), None, 0, ctypes.byref(nc),
                                None, 0, ctypes.byref(nw)))
    chunks = np.zeros(nc.value, CHUNK_DTYPE)
    work = np.zeros(nw.value, WORK_DTYPE)
    _check(lib().fcp_shard_plan(_np_ptr(sl), _np_ptr(cd), _np_ptr(br), len(sl), _np_ptr(chunks), nc.value,
                                ctypes.byref(nc), _np_ptr(work), nw.value, ctypes.byref(nw)))
    return chunks, work


def _spans(spans):
    """list of (seq, start, len) or a SPAN_DTYPE array -> contiguous SPAN_DTYPE array (order kept: the library
    checks it)"""
    if isinstance(spans, np.ndarray) and spans.dtype == SPAN_DTYPE:
        return np.ascontiguousarray(spans)
    a = np.zeros(len(spans), SPAN_DTYPE)
    for i, (k, st, ln) in enumerate(spans):
        a[i] = (k, st, ln)
    return a


def fcp_shard_plan_mixed(seq_lens, cp_degree, spans, base_rank=None):
    """Host only.  fcp_shard_plan for sequences with full-attention spans [(seq, start, len), ...]."""
    sl = np.ascontiguousarray(seq_lens, dtype=np.int32)
    cd = np.ascontiguousarray(cp_degree, dtype=np.int32)
    if sl.shape != cd.shape or sl.ndim != 1:
        raise ValueError("seq_lens and cp_degree must be 1-D and the same length")
    br = None if base_rank is None else np.ascontiguousarray(base_rank, dtype=np.int32)
    if br is not None and br.shape != sl.shape:
        raise ValueError("base_rank must match seq_lens")
    sp = _spans(spans)
    nc, nw = ctypes.c_int64(0), ctypes.c_int64(0)
    _check(lib().fcp_shard_plan_mixed(_np_ptr(sl), _np_ptr(cd), _np_ptr(br), len(sl), _np_ptr(sp), len(sp), None, 0,
                                      ctypes.byref(nc), None, 0, ctypes.byref(nw)))
    chunks = np.zeros(nc.value, CHUNK_DTYPE)
    work = np.zeros(nw.value, WORK_DTYPE)
    _check(lib().fcp_shard_plan_mixed(_np_ptr(sl), _np_ptr(cd), _np_ptr(br), len(sl), _np_ptr(sp), len(sp),
                                      _np_ptr(chunks), nc.value, ctypes.byref(nc), _np_ptr(work), nw.value,
                                      ctypes.byref(nw)))
    return chunks, work


def fcp_mask_tables(seq_lens, spans, chunks, rank):
    """Host only.  Returns (q_limit [tq of rank] int32, k_from [sum of seq_lens] int32, eta [n_seqs] float32)."""
    sl = np.ascontiguousarray(seq_lens, dtype=np.int32)
    sp = _spans(spans)
    ch = np.ascontiguousarray(chunks)
    if ch.dtype != CHUNK_DTYPE:
        raise ValueError("chunks must be a CHUNK_DTYPE array")
    nq = ctypes.c_int64(0)
    _check(lib().fcp_mask_tables(_np_ptr(sl), len(sl), _np_ptr(sp), len(sp), _np_ptr(ch), len(ch), int(rank), None, 0,
                                 ctypes.byref(nq), None, None))
    q_limit = np.zeros(nq.value, np.int32)
    k_from = np.zeros(int(sl.sum()), np.int32)
    eta = np.zeros(len(sl), np.float32)
    _check(lib().fcp_mask_tables(_np_ptr(sl), len(sl), _np_ptr(sp), len(sp), _np_ptr(ch), len(ch), int(rank),
                                 _np_ptr(q_limit), len(q_limit), ctypes.byref(nq), _np_ptr(k_from), _np_ptr(eta)))
    return q_limit, k_from, eta


class CostModel(ctypes.Structure):
    """fcp_cost_model: coefficients of the scheduler's time model (Eq. 8-9)."""
    _fields_ = [("alpha1", ctypes.c_double), ("alpha2", ctypes.c_double), ("beta1", ctypes.c_double),
                ("alpha3_over_v", ctypes.c_double), ("beta2", ctypes.c_double)]


def fcp_plan_groups(seq_lens, n_ranks, tokens_per_rank, cost_model, eta=None):
    """Host only.  Returns dict(group_of_seq, d_min, degree, base_rank, makespan); raises FcpError (capacity) if
    the groups' minimum degrees do not fit n_ranks.  cost_model: CostModel or a 5-tuple in its field order."""
    sl = np.ascontiguousarray(seq_lens, dtype=np.int32)
    if sl.ndim != 1:
        raise ValueError("seq_lens must be 1-D")
    et = None if eta is None else np.ascontiguousarray(eta, dtype=np.float32)
    if et is not None and et.shape != sl.shape:
        raise ValueError("eta must match seq_lens")
    cm = cost_model if isinstance(cost_model, CostModel) else CostModel(*[float(x) for x in cost_model])
    k = len(sl)
    group_of = np.zeros(k, np.int32)
    d_min, degree, base = (np.zeros(max(k, 1), np.int32) for _ in range(3))
    ng, mk = ctypes.c_int32(0), ctypes.c_double(0.0)
    _check(lib().fcp_plan_groups(_np_ptr(sl), _np_ptr(et), k, int(n_ranks), int(tokens_per_rank), ctypes.byref(cm),
                                 _np_ptr(group_of), ctypes.byref(ng), _np_ptr(d_min), _np_ptr(degree), _np_ptr(base),
                                 ctypes.byref(mk)))
    n = ng.value
    return {"group_of_seq": group_of, "d_min": d_min[:n].copy(), "degree": degree[:n].copy(),
            "base_rank": base[:n].copy(), "makespan": mk.value}


def fcp_group_shard_args(group_of_seq, group_degree, group_base_rank):
    """Host only.  (cp_degree, base_rank) per sequence for fcp_shard_plan: every sequence at its group's degree."""
    go = np.ascontiguousarray(group_of_seq, dtype=np.int32)
    gd = np.ascontiguousarray(group_degree, dtype=np.int32)
    gb = np.ascontiguousarray(group_base_rank, dtype=np.int32)
    if gd.shape != gb.shape or go.ndim != 1 or gd.ndim != 1:
        raise ValueError("group_degree and group_base_rank must be 1-D and the same length")
    cd, br = np.zeros(len(go), np.int32), np.zeros(len(go), np.int32)
    _check(lib().fcp_group_shard_args(_np_ptr(go), len(go), _np_ptr(gd), _np_ptr(gb), len(gd), _np_ptr(cd), _np_ptr(br)))
    return cd, br


def fcp_scratch_bytes(which, tq, tkv, hq, hkv, head_dim, n_work, n_parts) -> int:
    return int(lib().fcp_scratch_bytes(which, tq, tkv, hq, hkv, head_dim, n_work, n_parts))


def fcp_attn_fwd_step(q, k, v, cu_seqlens_kv, work, n_parts, softmax_scale, o_part, lse_part, scratch, stream=None):
    """q [tq,hq,D], k/v [tkv,hkv,D] bf16; cu_seqlens_kv int32 [n_seqs+1]; work: uint8 device tensor
    holding fcp_work_desc records; o_part [n_parts,tq,hq,D] fp32; lse_part [n_parts,hq,tq] fp32."""
    tq, hq, D = q.shape
    tkv, hkv, _ = k.shape
    n_work = work.numel() // WORK_DTYPE.itemsize
    _check(lib().fcp_attn_fwd_step(_dev_ptr(q), _dev_ptr(k), _dev_ptr(v), _dev_ptr(cu_seqlens_kv),
                                   cu_seqlens_kv.numel() - 1, _dev_ptr(work), n_work, n_parts, tq, tkv, hq, hkv, D,
                                   float(softmax_scale), _dev_ptr(o_part), _dev_ptr(lse_part), _dev_ptr(scratch),
                                   scratch.numel() * scratch.element_size(), _stream(stream)))


def fcp_attn_fwd_step_static(q, k, v, cu_seqlens_kv, work, n_parts, softmax_scale, o_part, lse_part, stream=None):
    """fcp_attn_fwd_step with the library's static work area (no scratch argument, no allocation)."""
    tq, hq, D = q.shape
    tkv, hkv, _ = k.shape
    n_work = work.numel() // WORK_DTYPE.itemsize
    _check(lib().fcp_attn_fwd_step_static(_dev_ptr(q), _dev_ptr(k), _dev_ptr(v), _dev_ptr(cu_seqlens_kv),
                                          cu_seqlens_kv.numel() - 1, _dev_ptr(work), n_work, n_parts, tq, tkv, hq, hkv, D,
                                          float(softmax_scale), _dev_ptr(o_part), _dev_ptr(lse_part), _stream(stream)))


def fcp_attn_fwd_step_mixed(q, k, v, cu_seqlens_kv, work, n_parts, softmax_scale, q_limit, o_part, lse_part, scratch,
                            stream=None):
    """fcp_attn_fwd_step under a mixed mask; q_limit: int32 device tensor [tq]."""
    tq, hq, D = q.shape
    tkv, hkv, _ = k.shape
    if q_limit.numel() != tq:
        raise ValueError("q_limit must have one entry per local query row")
    n_work = work.numel() // WORK_DTYPE.itemsize
    _check(lib().fcp_attn_fwd_step_mixed(_dev_ptr(q), _dev_ptr(k), _dev_ptr(v), _dev_ptr(cu_seqlens_kv),
                                         cu_seqlens_kv.numel() - 1, _dev_ptr(work), n_work, n_parts, tq, tkv, hq, hkv, D,
                                         float(softmax_scale), _dev_ptr(q_limit), _dev_ptr(o_part), _dev_ptr(lse_part),
                                         _dev_ptr(scratch), scratch.numel() * scratch.element_size(), _stream(stream)))


def fcp_attn_fwd_step_running(q, k, v, cu_seqlens_kv, work, softmax_scale, o_run, lse_run, scratch, o_out=None,
                              q_limit=None, stream=None):
    """One ring step merged into the running result (o_run [tq,hq,D] fp32, lse_run [hq,tq] fp32, in/out);
    o_out: optional bf16 [tq,hq,D]; q_limit: optional int32 [tq] (mixed mask)."""
    tq, hq, D = q.shape
    tkv, hkv, _ = k.shape
    n_work = work.numel() // WORK_DTYPE.itemsize
    _check(lib().fcp_attn_fwd_step_running(_dev_ptr(q), _dev_ptr(k), _dev_ptr(v), _dev_ptr(cu_seqlens_kv),
                                           cu_seqlens_kv.numel() - 1, _dev_ptr(work), n_work, tq, tkv, hq, hkv, D,
                                           float(softmax_scale), _dev_ptr(q_limit), _dev_ptr(o_run), _dev_ptr(lse_run),
                                           _dev_ptr(o_out), _dev_ptr(scratch), scratch.numel() * scratch.element_size(),
                                           _stream(stream)))


def fcp_lse_merge(o_part, lse_part, o, lse, stream=None):
    n_parts, tq, hq, D = o_part.shape
    _check(lib().fcp_lse_merge(_dev_ptr(o_part), _dev_ptr(lse_part), n_parts, tq, hq, D, _dev_ptr(o), _dev_ptr(lse),
                               _stream(stream)))


def fcp_attn_bwd_delta(o, d_o, delta, stream=None):
    tq, hq, D = o.shape
    _check(lib().fcp_attn_bwd_delta(_dev_ptr(o), _dev_ptr(d_o), tq, hq, D, _dev_ptr(delta), _stream(stream)))


def fcp_attn_bwd_step(q, k, v, d_o, lse, delta, cu_seqlens_kv, work, softmax_scale, dq_acc, dk_acc, dv_acc, scratch,
                      stream=None):
    tq, hq, D = q.shape
    tkv, hkv, _ = k.shape
    n_work = work.numel() // WORK_DTYPE.itemsize
    _check(lib().fcp_attn_bwd_step(_dev_ptr(q), _dev_ptr(k), _dev_ptr(v), _dev_ptr(d_o), _dev_ptr(lse), _dev_ptr(delta),
                                   _dev_ptr(cu_seqlens_kv), cu_seqlens_kv.numel() - 1, _dev_ptr(work), n_work, tq, tkv,
                                   hq, hkv, D, float(softmax_scale), _dev_ptr(dq_acc), _dev_ptr(dk_acc), _dev_ptr(dv_acc),
                                   _dev_ptr(scratch), scratch.numel() * scratch.element_size(), _stream(stream)))


def fcp_attn_bwd_step_mixed(q, k, v, d_o, lse, delta, cu_seqlens_kv, work, softmax_scale, q_limit, k_from, dq_acc, dk_acc,
                            dv_acc, scratch, stream=None):
    """fcp_attn_bwd_step under a mixed mask; q_limit [tq], k_from [tkv]: int32 device tensors."""
    tq, hq, D = q.shape
    tkv, hkv, _ = k.shape
    if q_limit.numel() != tq or k_from.numel() != tkv:
        raise ValueError("q_limit / k_from must have one entry per local query row / pool row")
    n_work = work.numel() // WORK_DTYPE.itemsize
    _check(lib().fcp_attn_bwd_step_mixed(_dev_ptr(q), _dev_ptr(k), _dev_ptr(v), _dev_ptr(d_o), _dev_ptr(lse),
                                         _dev_ptr(delta), _dev_ptr(cu_seqlens_kv), cu_seqlens_kv.numel() - 1,
                                         _dev_ptr(work), n_work, tq, tkv, hq, hkv, D, float(softmax_scale),
                                         _dev_ptr(q_limit), _dev_ptr(k_from), _dev_ptr(dq_acc), _dev_ptr(dk_acc),
                                         _dev_ptr(dv_acc), _dev_ptr(scratch), scratch.numel() * scratch.element_size(),
                                         _stream(stream)))


def fcp_attn_fwd_step_direct(q, k, v, cu_seqlens_kv, work, n_parts, softmax_scale, o_part, lse_part, o, lse, scratch,
                             q_limit=None, stream=None):
    """Whole forward of a rank: rows fed by one work item get their final O / LSE at once (see include/fcp.h)."""
    tq, hq, D = q.shape
    tkv, hkv, _ = k.shape
    n_work = work.numel() // WORK_DTYPE.itemsize
    _check(lib().fcp_attn_fwd_step_direct(_dev_ptr(q), _dev_ptr(k), _dev_ptr(v), _dev_ptr(cu_seqlens_kv),
                                          cu_seqlens_kv.numel() - 1, _dev_ptr(work), n_work, int(n_parts), tq, tkv, hq, hkv,
                                          D, float(softmax_scale), _dev_ptr(q_limit), _dev_ptr(o_part), _dev_ptr(lse_part),
                                          _dev_ptr(o), _dev_ptr(lse), _dev_ptr(scratch),
                                          scratch.numel() * scratch.element_size(), _stream(stream)))


def fcp_lse_merge_direct(o_part, lse_part, o, lse, tkv, scratch, n_work, stream=None):
    """Second half of the direct forward: merges the rows that have partial results."""
    n_parts, tq, hq, D = o_part.shape
    _check(lib().fcp_lse_merge_direct(_dev_ptr(o_part), _dev_ptr(lse_part), n_parts, tq, int(tkv), hq, D, _dev_ptr(o),
                                      _dev_ptr(lse), _dev_ptr(scratch), int(n_work), _stream(stream)))


def fcp_attn_bwd_step_direct(q, k, v, d_o, lse, delta, cu_seqlens_kv, work, softmax_scale, dq_acc, dk_acc, dv_acc,
                             dq_out, dk_out, dv_out, scratch, q_limit=None, k_from=None, stream=None):
    """Whole backward of a rank: rows owned by one unit are written to the bf16 outputs at once (see include/fcp.h)."""
    tq, hq, D = q.shape
    tkv, hkv, _ = k.shape
    n_work = work.numel() // WORK_DTYPE.itemsize
    _check(lib().fcp_attn_bwd_step_direct(_dev_ptr(q), _dev_ptr(k), _dev_ptr(v), _dev_ptr(d_o), _dev_ptr(lse),
                                          _dev_ptr(delta), _dev_ptr(cu_seqlens_kv), cu_seqlens_kv.numel() - 1,
                                          _dev_ptr(work), n_work, tq, tkv, hq, hkv, D, float(softmax_scale),
                                          _dev_ptr(q_limit), _dev_ptr(k_from), _dev_ptr(dq_acc), _dev_ptr(dk_acc),
                                          _dev_ptr(dv_acc), _dev_ptr(dq_out), _dev_ptr(dk_out), _dev_ptr(dv_out),
                                          _dev_ptr(scratch), scratch.numel() * scratch.element_size(), _stream(stream)))


def fcp_grad_finalize_direct(dq_acc, dk_acc, dv_acc, dq_out, dk_out, dv_out, scratch, n_work, stream=None):
    """Second half of the direct backward: converts the accumulated rows, zeroes the untouched ones."""
    tq, hq, D = dq_acc.shape
    tkv, hkv, _ = dk_acc.shape
    _check(lib().fcp_grad_finalize_direct(_dev_ptr(dq_acc), _dev_ptr(dk_acc), _dev_ptr(dv_acc), _dev_ptr(dq_out),
                                          _dev_ptr(dk_out), _dev_ptr(dv_out), _dev_ptr(scratch), int(n_work), tq, tkv, hq,
                                          hkv, D, _stream(stream)))


def fcp_grad_finalize(acc, out_bf16, stream=None):
    _check(lib().fcp_grad_finalize(_dev_ptr(acc), _dev_ptr(out_bf16), acc.numel(), _stream(stream)))


def fcp_scratch_status(scratch, stream=None):
    """(n_tiles, n_rejected) recorded by the last step that used `scratch`; synchronises."""
    a, b = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(lib().fcp_scratch_status(_dev_ptr(scratch), _stream(stream), ctypes.byref(a), ctypes.byref(b)))
    return a.value, b.value
