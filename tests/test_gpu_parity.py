"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle, element by
element, on seeded inputs that span several tiles, ragged tails and every CP degree 1..8."""
import numpy as np
import pytest

import fcp_synth as synth
from oracle import attn as oattn

from parity import TOL_BF16_REL, check_rank, rel_err

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def test_cfg0_single_sequence_d64_forward():
    wl = synth.make_workload(0)
    q, k, v, do = synth.draw_qkvdo(wl)
    _say("cfg0 L=512 d=1 h4x4 D=64 fwd")
    res = check_rank(wl, q, k, v, None, 0, backward=False, check_partials=True, label="cfg0")
    _say(f"  {res}")


def test_cfg1_L4096_degree3_rank1_fwd_bwd():
    wl = synth.make_workload(1)
    q, k, v, do = synth.draw_qkvdo(wl)
    _say("cfg1 L=4096 d=3 rank1 h8x8 D=128 fwd+bwd")
    res = check_rank(wl, q, k, v, do, 1, backward=True, check_partials=True, label="cfg1")
    _say("  " + str({a: b for a, b in res.items() if not a.startswith("_")}))


@pytest.mark.parametrize("d", range(1, 9))
def test_every_degree_all_ranks(d):
    """One odd-length sequence at degree d packed with a short degree-1 sequence; every rank is
    checked, and the ranks' dK/dV partial sums add up to the unsharded gradient."""
    L = 997 + 13 * d
    wl = synth.custom_workload([L, 75], [d, 1], hq=4, hkv=2, head_dim=128, seed=100 + d)
    q, k, v, do = synth.draw_qkvdo(wl)
    dK_sum = dV_sum = None
    for r in range(d):
        _say(f"degree {d} rank {r} L={L}")
        res = check_rank(wl, q, k, v, do, r, backward=True, check_partials=(r == d - 1), label=f"d{d}r{r}")
        dK_sum = res["_dK_acc"] if dK_sum is None else dK_sum + res["_dK_acc"]
        dV_sum = res["_dV_acc"] if dV_sum is None else dV_sum + res["_dV_acc"]
    _, dK_ref, dV_ref = oattn.attn_bwd(q, k, v, do, wl.cu_seqlens, wl.softmax_scale)
    assert rel_err(dK_sum, dK_ref) <= TOL_BF16_REL and rel_err(dV_sum, dV_ref) <= TOL_BF16_REL


@pytest.mark.parametrize("hq,hkv,D", [(10, 2, 128), (4, 4, 64), (6, 2, 64), (8, 1, 128)])
def test_head_layouts(hq, hkv, D):
    """Grouped heads incl. ratio 5 (not a power of two), head counts that are / are not a
    multiple of 8, both head dims."""
    wl = synth.custom_workload([300, 1, 129, 64, 517], [2, 1, 1, 1, 3], hq=hq, hkv=hkv, head_dim=D, seed=7)
    q, k, v, do = synth.draw_qkvdo(wl)
    for r in range(3):
        _say(f"heads {hq}/{hkv} D={D} rank {r}")
        check_rank(wl, q, k, v, do, r, backward=True, check_partials=True, label=f"h{hq}x{hkv}D{D}r{r}")


def test_degenerate_lengths():
    """Length 1, lengths below 2d (empty chunks), exact tile multiples, tile multiple +- 1."""
    lens = [1, 5, 128, 127, 129, 64, 65, 3, 256, 2]
    deg = [1, 4, 1, 1, 2, 1, 1, 2, 2, 1]
    wl = synth.custom_workload(lens, deg, hq=8, hkv=2, head_dim=128, seed=21)
    q, k, v, do = synth.draw_qkvdo(wl)
    for r in range(4):
        _say(f"degenerate lengths rank {r}")
        check_rank(wl, q, k, v, do, r, backward=True, check_partials=True, label=f"degenerate r{r}")


def test_many_short_sequences():
    rng = np.random.default_rng(5)
    lens = rng.integers(1, 200, size=40)
    wl = synth.custom_workload(lens, np.ones(40, np.int32), hq=8, hkv=8, head_dim=128, seed=22)
    q, k, v, do = synth.draw_qkvdo(wl)
    _say("40 short sequences, degree 1")
    check_rank(wl, q, k, v, do, 0, backward=True, label="shorts")


def test_cfg2_full_size_sampled():
    """The 32K-token packed workload in the launch configuration bench.py times (rank 0, 32 query / 8 KV heads,
    D = 128).  The oracle cannot redo all of it in seconds, so: O, LSE and dQ of every 61st row of the rank for
    the query heads of KV heads 0 and 5, and dK, dV of those two KV heads in full (their query heads, every row
    of the rank) - heads are independent, so a head subset is the exact result for those heads.  Both the plain and
    the direct entry points are held against the oracle on these samples."""
    import torch
    from paper_2602_21788_amd.rank import RankAttention
    from oracle import plan as oplan
    from parity import TOL_LSE_ABS, bf16_tensor_to_f64
    wl = synth.make_workload(2)
    q, k, v, do = synth.draw_qkvdo(wl)
    _say(f"cfg2 {wl.name} rank {wl.rank}: full-size run, sampled comparison")
    ra = RankAttention(wl.seq_lens, wl.cp_degree, wl.rank, wl.hq, wl.hkv, wl.head_dim, wl.softmax_scale)
    ra.set_inputs(q, k, v, do)
    ra.forward()
    ra.backward()
    torch.cuda.synchronize()
    ochunks, _ = oplan.shard_plan(wl.seq_lens, wl.cp_degree)
    rows = oplan.rank_rows(ochunks, wl.cu_seqlens, wl.rank)
    assert len(rows) == ra.tq
    O = bf16_tensor_to_f64(ra.o)
    LSE = ra.lse.cpu().numpy().astype(np.float64).T
    dQ, dK, dV = (bf16_tensor_to_f64(x) for x in (ra.dq, ra.dk, ra.dv))
    for x in (O, LSE, dQ, dK, dV):
        assert np.isfinite(x).all()
    # The direct forward (what bench.py times) on poisoned buffers: every element against partial results + merge.
    for t in (ra.o, ra.lse, ra.o_part, ra.lse_part):
        t.fill_(float("nan"))
    ra.forward_direct()
    torch.cuda.synchronize()
    O_d, LSE_d = bf16_tensor_to_f64(ra.o), ra.lse.cpu().numpy().astype(np.float64).T
    assert np.isfinite(O_d).all() and np.isfinite(LSE_d).all()
    assert rel_err(O_d, O) <= 2.0 ** -7 and np.abs(LSE_d - LSE).max() <= 1e-5
    # The direct backward (what bench.py times) on poisoned buffers: every element against the accumulating path,
    # which is checked against the oracle below - the arithmetic is the same up to the order of the fp32 atomics.
    for t in (ra.dq_acc, ra.dk_acc, ra.dv_acc, ra.dq, ra.dk, ra.dv):
        t.fill_(float("nan"))
    ra.backward_direct()
    torch.cuda.synchronize()
    direct = {}
    for name, acc, x in (("dQ", dQ, ra.dq), ("dK", dK, ra.dk), ("dV", dV, ra.dv)):
        d = direct[name] = bf16_tensor_to_f64(x)
        assert np.isfinite(d).all(), name
        assert rel_err(d, acc) <= 2.0 ** -7, (name, "direct vs accumulating", rel_err(d, acc))
    G = wl.hq // wl.hkv
    sel = np.arange(0, len(rows), 61)
    for kvh in (0, 5):
        hs = slice(kvh * G, (kvh + 1) * G)
        qs, dos = np.ascontiguousarray(q[:, hs]), np.ascontiguousarray(do[:, hs])
        ks, vs = np.ascontiguousarray(k[:, kvh:kvh + 1]), np.ascontiguousarray(v[:, kvh:kvh + 1])
        O_ref, LSE_ref = oattn.attn_fwd(qs, ks, vs, wl.cu_seqlens, wl.softmax_scale, rows)
        assert rel_err(O[sel, hs], O_ref[sel]) <= TOL_BF16_REL
        assert np.abs(LSE[sel, hs] - LSE_ref[sel]).max() <= TOL_LSE_ABS
        dQ_ref = oattn.attn_dq(qs, ks, vs, dos, wl.cu_seqlens, wl.softmax_scale, rows[sel], O_ref[sel], LSE_ref[sel])
        assert rel_err(dQ[sel, hs], dQ_ref) <= TOL_BF16_REL
        dK_ref, dV_ref = oattn.attn_dkv(qs, ks, vs, dos, wl.cu_seqlens, wl.softmax_scale, rows, O_ref, LSE_ref)
        e = {"O": rel_err(O[sel, hs], O_ref[sel]), "dQ": rel_err(dQ[sel, hs], dQ_ref),
             "dK": rel_err(dK[:, kvh:kvh + 1], dK_ref), "dV": rel_err(dV[:, kvh:kvh + 1], dV_ref)}
        _say(f"  kv head {kvh}: {e}")
        assert e["dK"] <= TOL_BF16_REL and e["dV"] <= TOL_BF16_REL
        # the direct entry points (what bench.py times) against the oracle itself, the same samples
        ed = {"O": rel_err(O_d[sel, hs], O_ref[sel]), "LSE": float(np.abs(LSE_d[sel, hs] - LSE_ref[sel]).max()),
              "dQ": rel_err(direct["dQ"][sel, hs], dQ_ref), "dK": rel_err(direct["dK"][:, kvh:kvh + 1], dK_ref),
              "dV": rel_err(direct["dV"][:, kvh:kvh + 1], dV_ref)}
        _say(f"  kv head {kvh}, direct entry points: {ed}")
        assert ed["LSE"] <= TOL_LSE_ABS and all(ed[n] <= TOL_BF16_REL for n in ("O", "dQ", "dK", "dV")), ed


def test_planned_microbatch_atomic_groups_end_to_end():
    """Scheduler to kernels: fcp_plan_groups packs a micro-batch into atomic groups and gives them degrees, every
    sequence then runs at its GROUP's degree on the group's ranks (the paper's execution of an atomic group: short
    sequences are sharded too), fcp_shard_plan splits them, and every rank's attention matches the oracle; the ranks'
    dK/dV partial sums add up to the unsharded gradient."""
    import paper_2602_21788_amd as fcp
    lens = [3000, 700, 300, 260, 90, 40, 1500]
    n_ranks, cap = 6, 1024
    plan = fcp.fcp_plan_groups(lens, n_ranks, cap, (1e-9, 1e-7, 1e-5, 0.0, 0.0))
    deg, base = fcp.fcp_group_shard_args(plan["group_of_seq"], plan["degree"], plan["base_rank"])
    _say(f"planned micro-batch: groups {plan['group_of_seq'].tolist()} degrees {plan['degree'].tolist()} "
         f"-> per-sequence degree {deg.tolist()} base {base.tolist()}")
    assert plan["degree"].sum() <= n_ranks and deg[0] >= 3 and (deg[np.array(lens) < 100] > 1).any()
    wl = synth.custom_workload(lens, deg, hq=4, hkv=2, head_dim=128, seed=55)
    q, k, v, do = synth.draw_qkvdo(wl)
    dK_sum = dV_sum = None
    for r in range(int(plan["degree"].sum())):
        res = check_rank(wl, q, k, v, do, r, backward=True, check_partials=True, label=f"planned r{r}", base_rank=base)
        if res is None:
            continue
        dK_sum = res["_dK_acc"] if dK_sum is None else dK_sum + res["_dK_acc"]
        dV_sum = res["_dV_acc"] if dV_sum is None else dV_sum + res["_dV_acc"]
    _, dK_ref, dV_ref = oattn.attn_bwd(q, k, v, do, wl.cu_seqlens, wl.softmax_scale)
    assert rel_err(dK_sum, dK_ref) <= TOL_BF16_REL and rel_err(dV_sum, dV_ref) <= TOL_BF16_REL


def test_profiler_fits_measured_attention_times():
    """The scheduler's Profiler on this library's own kernels: fit Eq. 8's compute model to measured forward + backward
    times of single sequences and plan a micro-batch with it (the paper reports estimation errors below 8 %; the
    bound here is loose because short sequences are launch-bound)."""
    from paper_2602_21788_amd import profiler
    import paper_2602_21788_amd as fcp
    lens = [2048, 4096, 8192, 12288, 16384]
    times = profiler.profile_attention(lens, [1] * len(lens))
    (a1, a2, b1), err = profiler.fit_compute_coefficients(lens, [1] * len(lens), times)
    _say(f"profiler: times {['%.3f ms' % (t * 1e3) for t in times]} alpha1 {a1:.3e} alpha2 {a2:.3e} beta1 {b1:.3e} max rel err {err:.3f}")
    assert a1 > 0 and err < 0.25
    plan = fcp.fcp_plan_groups([16384, 4096, 4096, 2048], 8, 8192, (a1, max(a2, 0.0), max(b1, 0.0), 0.0, 0.0))
    assert plan["d_min"][0] == 2 and plan["degree"][0] >= plan["degree"][1] and sum(plan["degree"]) <= 8


@pytest.mark.parametrize("case", ["d3_packed", "d5_all_ranks", "shorts_D64", "mixed_mask"])
def test_running_merge_forward_equals_partial_plus_merge(case):
    """fcp_attn_fwd_step_running, one call per ring step with no partial results, against the oracle and against
    the partial + merge pair (same kernels, same tiles: O within one bf16 rounding, LSE to 1e-5)."""
    import torch
    from paper_2602_21788_amd.rank import RankAttention
    from oracle import plan as oplan
    from parity import TOL_LSE_ABS, bf16_tensor_to_f64
    spans = None
    if case == "d3_packed":
        wl = synth.custom_workload([2100, 75, 640], [3, 1, 2], hq=8, hkv=2, head_dim=128, seed=61); ranks = [0, 2]
    elif case == "d5_all_ranks":
        wl = synth.custom_workload([1777], [5], hq=4, hkv=4, head_dim=128, seed=62); ranks = range(5)
    elif case == "shorts_D64":
        wl = synth.custom_workload([1, 130, 64, 257, 33, 511], [1] * 6, hq=6, hkv=2, head_dim=64, seed=63); ranks = [0]
    else:
        wl = synth.custom_workload([1500, 300], [3, 1], hq=4, hkv=2, head_dim=128, seed=64); ranks = range(3)
        spans = [(0, 200, 330), (0, 700, 64), (0, 990, 30), (1, 10, 200)]
    q, k, v, do = synth.draw_qkvdo(wl)
    sid = None if spans is None else oplan.span_ids(wl.seq_lens, spans)
    ochunks, _ = oplan.shard_plan(wl.seq_lens, wl.cp_degree, spans=spans)
    for r in ranks:
        _say(f"running merge: {case} rank {r}")
        ra = RankAttention(wl.seq_lens, wl.cp_degree, r, wl.hq, wl.hkv, wl.head_dim, wl.softmax_scale, spans=spans)
        ra.set_inputs(q, k, v, do)
        ra.forward()
        torch.cuda.synchronize()
        o_ref_path, lse_ref_path = bf16_tensor_to_f64(ra.o), ra.lse.cpu().numpy().astype(np.float64)
        ra.forward_running()
        torch.cuda.synchronize()
        O, LSE = bf16_tensor_to_f64(ra.o), ra.lse.cpu().numpy().astype(np.float64)
        rows = oplan.rank_rows(ochunks, wl.cu_seqlens, r)
        O_ref, LSE_ref = oattn.attn_fwd(q, k, v, wl.cu_seqlens, wl.softmax_scale, rows, span_id=sid)
        assert np.isfinite(O).all() and np.isfinite(LSE).all()
        assert rel_err(O, O_ref) <= TOL_BF16_REL and np.abs(LSE.T - LSE_ref).max() <= TOL_LSE_ABS
        assert np.abs(LSE - lse_ref_path).max() <= 1e-5
        assert np.abs(O - o_ref_path).max() <= 2.0 ** -7 * max(1.0, np.abs(o_ref_path).max())
        assert rel_err(ra.o_run.cpu().numpy().astype(np.float64), O_ref) <= 1e-2     # the fp32 running result itself


@pytest.mark.parametrize("path", ["plain", "direct"])
def test_whole_path_in_a_hip_graph_replays_identically(path):
    """The library calls enqueue kernels only (no allocation, no host synchronisation, no memset nodes), so the whole
    path of a rank can be captured into a HIP graph.  The graph is replayed three times with eager work and
    synchronisations in between and fresh inputs before every replay; every replay must reproduce the eager result of
    the same inputs (bit for bit where no atomics are involved: O, LSE, dQ of exclusive rows; to 1e-6 relative for
    the fp32 accumulators that several work items add to)."""
    import torch
    from paper_2602_21788_amd.rank import RankAttention
    wl = synth.custom_workload([1300, 200, 650], [3, 1, 2], hq=8, hkv=2, head_dim=128, seed=71)
    ra = RankAttention(wl.seq_lens, wl.cp_degree, 0, wl.hq, wl.hkv, wl.head_dim, wl.softmax_scale)
    ra.set_random_inputs(seed=1)

    def whole_path():
        if path == "direct":           # (the entry points bench.py times: nothing cleared by the caller)
            ra.forward_direct()
            ra.backward_direct()
        else:
            ra.forward()
            ra.backward()

    whole_path()                       # eager warm-up: the kernels' LDS limits are raised outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        whole_path()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            whole_path()
    torch.cuda.synchronize()
    gen = torch.Generator(device=ra.device).manual_seed(123)
    for replay in range(3):
        for t in (ra.q, ra.k, ra.v, ra.d_o):      # new inputs in the same buffers
            t.copy_(torch.randn(t.shape, generator=gen, device=ra.device, dtype=torch.float32).to(torch.bfloat16))
        for t in (ra.o, ra.lse, ra.dq, ra.dk, ra.dv):
            t.fill_(7.0)
        if path == "direct":
            for t in (ra.o_part, ra.lse_part, ra.dq_acc, ra.dk_acc, ra.dv_acc):
                t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [x.clone() for x in (ra.o, ra.lse, ra.dq, ra.dk, ra.dv)]
        whole_path()                   # eager, same inputs
        torch.cuda.synchronize()
        want = [ra.o, ra.lse, ra.dq, ra.dk, ra.dv]
        _say(f"graph replay {replay}: max |diff| " + ", ".join(f"{(a.float() - b.float()).abs().max().item():.2e}" for a, b in zip(got, want)))
        assert torch.equal(got[0], want[0]) and torch.equal(got[1], want[1])
        for a, b in zip(got[2:], want[2:]):
            assert torch.isfinite(a.float()).all()
            assert (a.float() - b.float()).abs().max().item() <= 1e-2 * b.float().abs().max().item()


def test_direct_entry_points_equal_the_plain_ones_on_random_batches():
    """Seeded random packed batches (lengths 1 .. 1500, degrees 1 .. 5 with every rank in turn, several head layouts,
    every third batch with full-attention spans): the direct forward / backward on NaN-filled buffers against the
    plain entry points on the same device inputs, element by element.  The plain path is what the other tests hold
    against the oracle; this one is about the row classification (untouched / several items / one owner) agreeing
    with what the kernels do, for layouts no hand-written case has."""
    import torch
    from paper_2602_21788_amd.rank import RankAttention
    rng = np.random.default_rng(2024)
    layouts = [(8, 2, 128), (4, 4, 64), (6, 2, 64), (8, 1, 128), (2, 2, 128)]
    n_cases = 0
    for case in range(18):
        n_seq = int(rng.integers(1, 7))
        lens = [int(x) for x in rng.integers(1, 1500, n_seq)]
        deg = [int(min(rng.integers(1, 6), max(1, L // 2))) for L in lens]
        hq, hkv, D = layouts[case % len(layouts)]
        spans = None
        if case % 3 == 2:
            spans = []
            for s, L in enumerate(lens):
                if L >= 40:
                    a = int(rng.integers(0, L - 30))
                    spans.append((s, a, int(rng.integers(2, min(300, L - a)))))
            spans = spans or None
        rank = case % max(deg)
        ra = RankAttention(lens, deg, rank, hq, hkv, D, spans=spans)
        if ra.tq == 0:
            continue
        _say(f"random batch {case}: lens {lens} degrees {deg} rank {rank} heads {hq}/{hkv} D {D} spans {spans}")
        ra.set_random_inputs(case)
        ra.forward(); ra.backward()
        torch.cuda.synchronize()
        plain = [t.clone() for t in (ra.o, ra.lse, ra.dq, ra.dk, ra.dv)]
        for t in (ra.o, ra.lse, ra.o_part, ra.lse_part, ra.dq_acc, ra.dk_acc, ra.dv_acc, ra.dq, ra.dk, ra.dv):
            t.fill_(float("nan"))
        ra.forward_direct(); ra.backward_direct()
        torch.cuda.synchronize()
        for name, a, b in zip(("O", "LSE", "dQ", "dK", "dV"), plain, (ra.o, ra.lse, ra.dq, ra.dk, ra.dv)):
            a, b = a.double(), b.double()
            assert not torch.isnan(b).any(), (case, name)
            assert torch.equal(torch.isinf(a), torch.isinf(b)), (case, name)      # LSE = -inf for rows without keys
            fin = torch.isfinite(a)
            scale = float(a[fin].abs().max()) if fin.any() else 1.0
            err = float((a[fin] - b[fin]).abs().max()) / max(scale, 1e-30) if fin.any() else 0.0
            assert err <= (1e-5 if name == "LSE" else 2.0 ** -7), (case, name, err)
        n_cases += 1
    assert n_cases >= 12
