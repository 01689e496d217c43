"""CPU-only checks of libfcp.so: it loads, exports every declared symbol, the host shard plan
is bit-exact against the oracle's independent re-implementation, and argument errors are
reported before any device work."""
import ctypes
import os
import re

import numpy as np
import pytest

import fcp_synth as synth
from oracle import plan as oplan
from paper_2602_21788_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_exports_match_header():
    hdr = open(os.path.join(ROOT, "include", "fcp.h")).read()
    declared = set(re.findall(r"\b(fcp_[a-z_]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_descriptor_struct_sizes():
    assert B.CHUNK_DTYPE.itemsize == 24 and B.WORK_DTYPE.itemsize == 44
    assert B.CHUNK_DTYPE == oplan.CHUNK_DTYPE and B.WORK_DTYPE == oplan.WORK_DTYPE


@pytest.mark.parametrize("cfg", range(5))
def test_plan_bit_exact_workloads(cfg):
    wl = synth.make_workload(cfg)
    c, w = B.fcp_shard_plan(wl.seq_lens, wl.cp_degree)
    oc, ow = oplan.shard_plan(wl.seq_lens, wl.cp_degree)
    assert c.tobytes() == oc.tobytes()
    assert w.tobytes() == ow.tobytes()


def test_plan_bit_exact_random():
    rng = np.random.default_rng(0)
    for _ in range(200):
        n = int(rng.integers(1, 7))
        lens = rng.integers(1, 200, size=n)
        deg = rng.integers(1, 9, size=n)
        base = rng.integers(0, 5, size=n) if rng.random() < 0.5 else None
        c, w = B.fcp_shard_plan(lens, deg, base)
        oc, ow = oplan.shard_plan(lens, deg, base)
        assert c.tobytes() == oc.tobytes() and w.tobytes() == ow.tobytes(), (lens, deg, base)


def test_plan_all_small_lengths_and_degrees():
    for d in range(1, 9):
        for L in range(1, 70):
            c, w = B.fcp_shard_plan([L], [d])
            oc, ow = oplan.shard_plan([L], [d])
            assert c.tobytes() == oc.tobytes() and w.tobytes() == ow.tobytes(), (L, d)


def test_plan_errors_and_two_call_sizing():
    L = B.lib()
    sl = np.array([10, 0], np.int32); cd = np.array([1, 1], np.int32)
    nc, nw = ctypes.c_int64(), ctypes.c_int64()
    rc = L.fcp_shard_plan(sl.ctypes.data, cd.ctypes.data, None, 2, None, 0, ctypes.byref(nc), None, 0, ctypes.byref(nw))
    assert rc == B.FCP_ERR_INVALID_ARG and b"seq_lens[1]" in L.fcp_last_error()
    sl = np.array([10, 9], np.int32); cd = np.array([2, 0], np.int32)
    rc = L.fcp_shard_plan(sl.ctypes.data, cd.ctypes.data, None, 2, None, 0, ctypes.byref(nc), None, 0, ctypes.byref(nw))
    assert rc == B.FCP_ERR_INVALID_ARG
    cd = np.array([2, 1], np.int32)
    rc = L.fcp_shard_plan(sl.ctypes.data, cd.ctypes.data, None, 2, None, 0, ctypes.byref(nc), None, 0, ctypes.byref(nw))
    assert rc == 0 and nc.value == 5 and L.fcp_last_error() == b""
    small = np.zeros(2, B.CHUNK_DTYPE)
    rc = L.fcp_shard_plan(sl.ctypes.data, cd.ctypes.data, None, 2, small.ctypes.data, 2, ctypes.byref(nc), None, 0, ctypes.byref(nw))
    assert rc == B.FCP_ERR_CAPACITY and nc.value == 5
    rc = L.fcp_shard_plan(None, cd.ctypes.data, None, 2, None, 0, ctypes.byref(nc), None, 0, ctypes.byref(nw))
    assert rc == B.FCP_ERR_INVALID_ARG


def test_device_entry_points_reject_bad_arguments_on_host():
    """Argument checks come before any HIP call, so they can be exercised without a GPU."""
    L = B.lib()
    fake = ctypes.c_void_p(0x1000)     # never dereferenced: every call below must fail first
    assert L.fcp_attn_fwd_step(None, fake, fake, fake, 1, fake, 1, 1, 8, 8, 4, 4, 128, 0.1, fake, fake, fake, 1 << 20, None) == B.FCP_ERR_INVALID_ARG
    assert L.fcp_attn_fwd_step(fake, fake, fake, fake, 1, fake, 1, 1, 8, 8, 4, 4, 96, 0.1, fake, fake, fake, 1 << 20, None) == B.FCP_ERR_UNSUPPORTED
    assert b"head_dim" in L.fcp_last_error()
    assert L.fcp_attn_fwd_step(fake, fake, fake, fake, 1, fake, 1, 1, 8, 8, 6, 4, 128, 0.1, fake, fake, fake, 1 << 20, None) == B.FCP_ERR_UNSUPPORTED
    assert L.fcp_attn_fwd_step(fake, fake, fake, fake, 1, fake, 1, 1, 8, 8, 4, 4, 128, 0.1, fake, fake, fake, 8, None) == B.FCP_ERR_CAPACITY
    assert L.fcp_attn_fwd_step(fake, fake, fake, fake, 1, fake, 1, 1, 8, 8, 4, 4, 128, -1.0, fake, fake, fake, 1 << 20, None) == B.FCP_ERR_INVALID_ARG
    assert L.fcp_attn_bwd_step(fake, fake, fake, fake, fake, fake, fake, 1, fake, 1, 8, 8, 4, 4, 32, 0.1, fake, fake, fake, fake, 1 << 20, None) == B.FCP_ERR_UNSUPPORTED
    assert L.fcp_attn_bwd_step(fake, fake, fake, fake, None, fake, fake, 1, fake, 1, 8, 8, 4, 4, 128, 0.1, fake, fake, fake, fake, 1 << 20, None) == B.FCP_ERR_INVALID_ARG
    # a rank whose bf16 Q rows pass 2^31 bytes (32-bit offsets inside a work item) is refused, one just below is not
    # refused for its size (it fails later, on the scratch size given here)
    assert L.fcp_attn_bwd_step(fake, fake, fake, fake, fake, fake, fake, 1, fake, 1, 1 << 18, 1 << 18, 32, 8, 128, 0.1, fake, fake, fake, fake, 1 << 40, None) == B.FCP_ERR_UNSUPPORTED
    assert b"2^30" in L.fcp_last_error()
    assert L.fcp_attn_bwd_step(fake, fake, fake, fake, fake, fake, fake, 1, fake, 1, 1 << 17, 1 << 17, 32, 8, 128, 0.1, fake, fake, fake, fake, 8, None) == B.FCP_ERR_CAPACITY
    assert L.fcp_lse_merge(fake, fake, 17, 8, 4, 128, fake, fake, None) == B.FCP_ERR_UNSUPPORTED
    assert L.fcp_lse_merge(fake, fake, 0, 8, 4, 128, fake, fake, None) == B.FCP_ERR_INVALID_ARG
    assert L.fcp_attn_bwd_delta(fake, None, 8, 4, 128, fake, None) == B.FCP_ERR_INVALID_ARG
    assert L.fcp_grad_finalize(fake, fake, -1, None) == B.FCP_ERR_INVALID_ARG
    assert L.fcp_scratch_bytes(B.FCP_SCRATCH_FWD, 1000, 1000, 4, 4, 128, 3, 2) > 64
    assert L.fcp_scratch_bytes(B.FCP_SCRATCH_BWD, 1000, 1000, 4, 4, 128, 3, 2) > 64
    # the direct entry points: outputs are required, the mask tables go together, long work lists are refused
    big = 1 << 30
    assert L.fcp_attn_fwd_step_direct(fake, fake, fake, fake, 1, fake, 1, 1, 8, 8, 4, 4, 128, 0.1, None, fake, fake, None, fake, fake, big, None) == B.FCP_ERR_INVALID_ARG
    assert L.fcp_attn_fwd_step_direct(fake, fake, fake, fake, 1, fake, 2000, 1, 8, 8, 4, 4, 128, 0.1, None, fake, fake, fake, fake, fake, big, None) == B.FCP_ERR_UNSUPPORTED
    assert b"direct mode" in L.fcp_last_error()
    assert L.fcp_lse_merge_direct(fake, fake, 1, 8, 8, 4, 128, fake, fake, None, 1, None) == B.FCP_ERR_INVALID_ARG
    bwd = lambda **kw: L.fcp_attn_bwd_step_direct(fake, fake, fake, fake, fake, fake, fake, 1, fake, kw.get("n_work", 1), 8, 8, 4, 4, 128, 0.1,
                                                 kw.get("q_limit"), None, fake, fake, fake, kw.get("dq_out", fake), fake, fake, fake, big, None)
    assert bwd(dq_out=None) == B.FCP_ERR_INVALID_ARG
    assert bwd(q_limit=fake) == B.FCP_ERR_INVALID_ARG and b"go together" in L.fcp_last_error()
    assert bwd(n_work=2000) == B.FCP_ERR_UNSUPPORTED and b"direct mode" in L.fcp_last_error()
    assert L.fcp_grad_finalize_direct(fake, fake, fake, fake, fake, None, fake, 1, 8, 8, 4, 4, 128, None) == B.FCP_ERR_INVALID_ARG
    assert L.fcp_grad_finalize_direct(fake, fake, fake, fake, fake, fake, fake, 1, 8, 8, 4, 4, 96, None) == B.FCP_ERR_UNSUPPORTED


def test_no_oracle_in_product_path():
    """The package must not import or reference the oracle."""
    pkg = os.path.join(ROOT, "paper_2602_21788_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".h")):
                txt = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in txt.lower(), f
