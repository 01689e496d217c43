"""Pins for the mixed-mask side of the oracle (CPU only).

The paper (Sec. 4.3, time estimation before Eq. 8) says only that multimodal models give some tokens
full attention and that a mask efficiency factor eta_k, determined by the shape of the mask, scales the
quadratic cost.  The reading taken: marked token spans attend in both directions inside the span, every
other pair is causal.  The paper prints no example, so the oracle is pinned to what that definition and
the mathematics fix:
  * no spans = the causal oracle, bit for bit; one span over the whole sequence = unmasked softmax
    (numpy by hand, torch float64 SDPA with autograd);
  * an explicit dense L x L masked softmax whose mask is built another way (lower triangle OR block
    diagonal of the spans), forward and all three gradients; finite differences;
  * the visible set of a row is a prefix 0..q_limit, the viewers of a key a suffix k_from..L-1 (what the
    kernels rely on), against closed forms of both tables;
  * eta in closed form; pairs of all ranks add up to the closed-form pair count;
  * the shard plan covers every visible pair exactly once, and the merged partials of its work items
    equal the unsharded attention.
"""
import numpy as np
import pytest
import torch

import fcp_synth as synth
from oracle import attn as oattn
from oracle import plan as oplan


def _rand_bits(rng, shape, scale=1.0):
    return synth.f32_to_bf16_bits((scale * rng.standard_normal(shape)).astype(np.float32))


def _block_mask(L, spans_of_seq):
    """lower triangle OR the spans' diagonal blocks"""
    m = np.tril(np.ones((L, L), bool))
    for st, ln in spans_of_seq:
        m[st:st + ln, st:st + ln] = True
    return m


def _dense_reference(q, k, v, do, lens, spans, scale):
    qf, kf, vf, dof = (synth.bf16_bits_to_f64(x) for x in (q, k, v, do))
    T, hq, D = qf.shape
    hkv = kf.shape[1]
    G = hq // hkv
    cu = np.concatenate([[0], np.cumsum(lens)])
    O = np.zeros_like(qf); LSE = np.zeros((T, hq))
    dQ = np.zeros_like(qf); dK = np.zeros_like(kf); dV = np.zeros_like(vf)
    for n, L in enumerate(lens):
        a, b = cu[n], cu[n + 1]
        mask = _block_mask(L, [(st, ln) for (s, st, ln) in spans if s == n])
        for h in range(hq):
            g = h // G
            S = scale * qf[a:b, h] @ kf[a:b, g].T
            E = np.where(mask, np.exp(S), 0.0)
            Z = E.sum(1, keepdims=True)
            P = E / Z
            O[a:b, h] = P @ vf[a:b, g]
            LSE[a:b, h] = np.log(Z[:, 0])
            dP = dof[a:b, h] @ vf[a:b, g].T
            dS = P * (dP - (dP * P).sum(1, keepdims=True))
            dQ[a:b, h] = scale * dS @ kf[a:b, g]
            dK[a:b, g] += scale * dS.T @ qf[a:b, h]
            dV[a:b, g] += P.T @ dof[a:b, h]
    return O, LSE, dQ, dK, dV


def _draw(rng, lens, hq, hkv, D):
    T = int(np.sum(lens))
    return (_rand_bits(rng, (T, hq, D)), _rand_bits(rng, (T, hkv, D)), _rand_bits(rng, (T, hkv, D)),
            _rand_bits(rng, (T, hq, D)))


LENS = [1, 7, 32, 13, 20]
SPANS = [(1, 2, 4), (2, 0, 5), (2, 10, 1), (2, 20, 12), (4, 3, 17)]   # (seq, start, length)


def test_no_spans_is_the_causal_oracle_bit_for_bit():
    rng = np.random.default_rng(0)
    q, k, v, do = _draw(rng, LENS, 4, 2, 8)
    cu = np.concatenate([[0], np.cumsum(LENS)]).astype(np.int32)
    none = np.full(int(cu[-1]), -1, np.int32)
    a = oattn.attn_fwd(q, k, v, cu, 0.3) + oattn.attn_bwd(q, k, v, do, cu, 0.3)
    b = oattn.attn_fwd(q, k, v, cu, 0.3, span_id=none) + oattn.attn_bwd(q, k, v, do, cu, 0.3, span_id=none)
    for x, y in zip(a, b):
        assert x.tobytes() == y.tobytes()


@pytest.mark.parametrize("hq,hkv,D", [(4, 4, 8), (6, 2, 16)])
def test_dense_matrix_with_block_mask(hq, hkv, D):
    rng = np.random.default_rng(1)
    q, k, v, do = _draw(rng, LENS, hq, hkv, D)
    cu = np.concatenate([[0], np.cumsum(LENS)]).astype(np.int32)
    sid = oplan.span_ids(LENS, SPANS)
    scale = 1.0 / np.sqrt(D)
    O, LSE = oattn.attn_fwd(q, k, v, cu, scale, span_id=sid)
    dQ, dK, dV = oattn.attn_bwd(q, k, v, do, cu, scale, span_id=sid)
    ref = _dense_reference(q, k, v, do, LENS, SPANS, scale)
    for got, r in zip((O, LSE, dQ, dK, dV), ref):
        np.testing.assert_allclose(got, r, rtol=1e-11, atol=1e-12)
    # and it is NOT the causal result (a mask argument that is ignored would pass the test above with spans = [])
    O_c, _ = oattn.attn_fwd(q, k, v, cu, scale)
    assert np.abs(O - O_c).max() > 1e-3


def test_whole_sequence_span_is_unmasked_attention_torch():
    """One span over the whole sequence: torch float64 SDPA without a mask, gradients by autograd."""
    rng = np.random.default_rng(2)
    L, hq, hkv, D = 37, 4, 2, 16
    q, k, v, do = _draw(rng, [L], hq, hkv, D)
    cu = np.array([0, L], np.int32)
    sid = oplan.span_ids([L], [(0, 0, L)])
    scale = 0.21
    O, LSE = oattn.attn_fwd(q, k, v, cu, scale, span_id=sid)
    dQ, dK, dV = oattn.attn_bwd(q, k, v, do, cu, scale, span_id=sid)
    tq, tk, tv, tdo = (torch.from_numpy(synth.bf16_bits_to_f64(x)).permute(1, 0, 2).clone() for x in (q, k, v, do))
    tq.requires_grad_(True); tk.requires_grad_(True); tv.requires_grad_(True)
    G = hq // hkv
    out = torch.nn.functional.scaled_dot_product_attention(tq, tk.repeat_interleave(G, 0), tv.repeat_interleave(G, 0),
                                                           is_causal=False, scale=scale)
    (out * tdo).sum().backward()
    np.testing.assert_allclose(O, out.detach().permute(1, 0, 2).numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dQ, tq.grad.permute(1, 0, 2).numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(dK, tk.grad.permute(1, 0, 2).numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(dV, tv.grad.permute(1, 0, 2).numpy(), rtol=1e-9, atol=1e-11)
    S = scale * np.einsum("ihc,jhc->hij", synth.bf16_bits_to_f64(q), np.repeat(synth.bf16_bits_to_f64(k), G, 1))
    np.testing.assert_allclose(LSE.T, np.log(np.exp(S).sum(2)), rtol=1e-12)


def test_constant_values_closed_form():
    """Equal keys inside a span: every row of the span averages ALL values of prefix + span,
    LSE = score + ln(number of visible keys)."""
    L, D, st, ln = 12, 8, 4, 5
    rng = np.random.default_rng(3)
    q = _rand_bits(rng, (L, 1, D))
    k = np.repeat(_rand_bits(rng, (1, 1, D)), L, 0)
    v = _rand_bits(rng, (L, 1, D))
    cu = np.array([0, L], np.int32)
    sid = oplan.span_ids([L], [(0, st, ln)])
    O, LSE = oattn.attn_fwd(q, k, v, cu, 0.5, span_id=sid)
    vf, qf, kf = (synth.bf16_bits_to_f64(x) for x in (v, q, k))
    for i in range(L):
        n_vis = st + ln if st <= i < st + ln else i + 1
        np.testing.assert_allclose(O[i, 0], vf[:n_vis, 0].mean(0), rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(LSE[i, 0], 0.5 * qf[i, 0] @ kf[0, 0] + np.log(n_vis), rtol=1e-12)


def test_finite_differences_with_spans():
    """The oracle's gradients against central difference quotients of the loss sum(O * dO), the loss evaluated in
    fp64 with a dense masked softmax around the (bf16-exact) inputs; one element of dQ and dV, two of dK."""
    rng = np.random.default_rng(4)
    lens, spans = [11], [(0, 3, 6)]
    q, k, v, do = _draw(rng, lens, 2, 1, 4)
    cu = np.array([0, 11], np.int32)
    sid = oplan.span_ids(lens, spans)
    scale = 0.4
    dQ, dK, dV = oattn.attn_bwd(q, k, v, do, cu, scale, span_id=sid)
    qf, kf, vf, dof = (synth.bf16_bits_to_f64(x) for x in (q, k, v, do))
    mask = _block_mask(11, [(3, 6)])

    def loss(qx, kx, vx):
        tot = 0.0
        for h in range(2):
            S = scale * qx[:, h] @ kx[:, 0].T
            E = np.where(mask, np.exp(S), 0.0)
            tot += ((E / E.sum(1, keepdims=True)) @ vx[:, 0] * dof[:, h]).sum()
        return tot

    eps = 1e-6
    for name, grad, idx in (("dQ", dQ, (5, 1, 2)), ("dK", dK, (7, 0, 1)), ("dV", dV, (4, 0, 3)), ("dK", dK, (8, 0, 0))):
        args = [qf.copy(), kf.copy(), vf.copy()]
        which = {"dQ": 0, "dK": 1, "dV": 2}[name]
        args[which][idx] += eps
        up = loss(*args)
        args[which][idx] -= 2 * eps
        dn = loss(*args)
        np.testing.assert_allclose(grad[idx], (up - dn) / (2 * eps), rtol=1e-6, atol=1e-8)


# ---- the interval form of the mask, eta, the plan --------------------------------------------------------------
def _random_spans(rng, lens, density=0.5):
    spans = []
    for k, L in enumerate(lens):
        pos = 0
        while pos < L:
            gap = int(rng.integers(0, max(2, L // 3)))
            ln = int(rng.integers(1, max(2, L // 2)))
            st = pos + gap
            if st >= L or rng.random() > density:
                break
            ln = min(ln, L - st)
            spans.append((k, st, ln))
            pos = st + ln
    return spans


def test_tables_are_intervals_with_closed_forms():
    rng = np.random.default_rng(5)
    for trial in range(20):
        lens = [int(x) for x in rng.integers(1, 40, size=4)]
        spans = _random_spans(rng, lens)
        chunks, _ = oplan.shard_plan(lens, [1] * len(lens), spans=spans)
        q_limit, k_from, eta = oplan.mask_tables(lens, spans, chunks, 0)
        sid = oplan.span_ids(lens, spans)
        cu = np.concatenate([[0], np.cumsum(lens)])
        for k, L in enumerate(lens):
            s = sid[cu[k]:cu[k + 1]]
            vis = oplan.visible_matrix(np.arange(L), np.arange(L), s, s)
            lim = q_limit[cu[k]:cu[k + 1]]                    # degree 1: local rows = pool rows
            frm = k_from[cu[k]:cu[k + 1]]
            for i in range(L):
                assert (vis[i] == (np.arange(L) <= lim[i])).all()       # a prefix
                assert (vis[:, i] == (np.arange(L) >= frm[i])).all()    # a suffix
            # closed forms: inside span [a, a+n) the limit is a+n-1 and the first viewer a; own position elsewhere
            want_lim, want_from = np.arange(L), np.arange(L)
            for (ks, a, n) in spans:
                if ks == k:
                    want_lim[a:a + n] = a + n - 1
                    want_from[a:a + n] = a
            assert (lim == want_lim).all() and (frm == want_from).all()
            assert (np.diff(lim) >= 0).all() and (np.diff(frm) >= 0).all()
            extra = sum(n * (n - 1) // 2 for (ks, a, n) in spans if ks == k)
            assert eta[k] == pytest.approx(extra / (L * (L + 1) // 2), abs=1e-15)


def _covered_pairs(work, rank, q_limit):
    """{(seq, q_pos, k_pos): times covered} from a rank's items with the per-row limit applied"""
    cnt = {}
    for w in work[work["rank"] == rank]:
        for r in range(int(w["q_len"])):
            lim = int(q_limit[int(w["q_local_off"]) + r])
            for sg in range(int(w["n_seg"])):
                for kp in range(int(w["k_seq_start"][sg]), int(w["k_seq_start"][sg]) + int(w["k_len"][sg])):
                    if kp <= lim:
                        key = (int(w["seq"]), int(w["q_seq_start"]) + r, kp)
                        cnt[key] = cnt.get(key, 0) + 1
    return cnt


@pytest.mark.parametrize("seed", range(6))
def test_plan_covers_every_visible_pair_once(seed):
    rng = np.random.default_rng(100 + seed)
    lens = [int(x) for x in rng.integers(1, 60, size=3)]
    degs = [int(x) for x in rng.integers(1, 5, size=3)]
    spans = _random_spans(rng, lens, density=0.8)
    chunks, work = oplan.shard_plan(lens, degs, spans=spans)
    sid = oplan.span_ids(lens, spans)
    cu = np.concatenate([[0], np.cumsum(lens)])
    total = 0
    for rank in range(max(degs)):
        q_limit, _, _ = oplan.mask_tables(lens, spans, chunks, rank)
        cnt = _covered_pairs(work, rank, q_limit)
        assert all(c == 1 for c in cnt.values())
        want = set()
        for ch in chunks[chunks["rank"] == rank]:
            k, L = int(ch["seq"]), lens[int(ch["seq"])]
            s = sid[cu[k]:cu[k + 1]]
            for qp in range(int(ch["seq_start"]), int(ch["seq_start"]) + int(ch["len"])):
                vis = oplan.visible_matrix([qp], np.arange(L), s[[qp]], s)[0]
                want |= {(k, qp, int(j)) for j in np.nonzero(vis)[0]}
        assert set(cnt) == want
        total += len(want)
    closed = sum(L * (L + 1) // 2 for L in lens) + sum(n * (n - 1) // 2 for (_, _, n) in spans)
    assert total == closed
    # every item has at least one visible pair in each of its segments (no empty segments are emitted)
    for w in work:
        q_limit, _, _ = oplan.mask_tables(lens, spans, chunks, int(w["rank"]))
        last = int(q_limit[int(w["q_local_off"]) + int(w["q_len"]) - 1])
        for sg in range(int(w["n_seg"])):
            assert int(w["k_seq_start"][sg]) <= last


def test_spans_none_plan_unchanged():
    lens, degs = [50, 9, 31], [3, 1, 2]
    a = oplan.shard_plan(lens, degs)
    b = oplan.shard_plan(lens, degs, spans=[])
    c = oplan.shard_plan(lens, degs, spans=[(0, 4, 1), (2, 30, 1)])     # spans of one token change nothing
    for x, y in ((a, b), (a, c)):
        assert x[0].tobytes() == y[0].tobytes() and x[1].tobytes() == y[1].tobytes()


def test_span_across_chunk_border_adds_a_later_segment():
    """L = 16 at degree 2: chunks [0,4) [4,8) [8,12) [12,16); a span [6, 10) makes chunk 1's rows 6, 7 see keys
    8, 9 of chunk 2, which a causal plan never pairs (chunk 2 is later)."""
    chunks, work = oplan.shard_plan([16], [2], spans=[(0, 6, 4)])
    causal = oplan.shard_plan([16], [2])[1]
    assert len(work) == len(causal) + 1 or any(int(w["n_seg"]) == 2 for w in work)
    hit = [w for w in work if int(w["q_seq_start"]) == 4 and 8 in [int(x) for x in w["k_seq_start"][:int(w["n_seg"])]]]
    assert len(hit) == 1 and int(hit[0]["rank"]) == 1       # chunk 1 belongs to rank 1; chunk 2 too: step 0


@pytest.mark.parametrize("degs", [[1, 1], [3, 2], [4, 1]])
def test_merged_partials_equal_unsharded_attention(degs):
    rng = np.random.default_rng(7)
    lens = [45, 23]
    spans = [(0, 5, 12), (0, 20, 9), (0, 40, 5), (1, 0, 8), (1, 15, 8)]
    hq, hkv, D = 4, 2, 8
    q, k, v, _ = _draw(rng, lens, hq, hkv, D)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    sid = oplan.span_ids(lens, spans)
    chunks, work = oplan.shard_plan(lens, degs, spans=spans)
    qf, kf, vf = (synth.bf16_bits_to_f64(x) for x in (q, k, v))
    for rank in range(max(degs)):
        rows = oplan.rank_rows(chunks, cu, rank)
        if len(rows) == 0:
            continue
        Op, Lp = oplan.rank_partials(qf, kf, vf, cu, chunks, work, rank, 0.35, span_id=sid)
        O, LSE = oplan.lse_merge(Op, Lp)
        O_ref, LSE_ref = oattn.attn_fwd(q, k, v, cu, 0.35, rows, span_id=sid)
        np.testing.assert_allclose(O, O_ref, rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(LSE, LSE_ref, rtol=1e-12)
