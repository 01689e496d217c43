"""Pins for the fp64 attention oracle (CPU only).

The oracle (oracle/attn_oracle.c) is the plain definition of paper Eq. 1 with the
causal mask of Sec. 4.3.  The paper prints no numeric example for attention, so the
oracle is pinned to what the mathematics fixes: closed forms, invariants, a library
routine on a special case (torch float64 SDPA + autograd), finite differences, and an
explicit dense softmax matrix on tiny inputs.  Each pin is chosen so that a dropped
term, a wrong sign, a wrong head mapping or a transposed operand breaks it.
"""
import numpy as np
import pytest
import torch

import fcp_synth as synth
from oracle import attn as oattn


def _rand_bits(rng, shape, scale=1.0):
    return synth.f32_to_bf16_bits((scale * rng.standard_normal(shape)).astype(np.float32))


def _dense_reference(q, k, v, do, cu, scale):
    """Explicit L x L masked softmax matrix per sequence and head, numpy fp64, with the
    gradients written as matrix products (independent formulation of the same maths)."""
    qf, kf, vf, dof = (synth.bf16_bits_to_f64(x) for x in (q, k, v, do))
    T, hq, D = qf.shape
    hkv = kf.shape[1]
    G = hq // hkv
    O = np.zeros_like(qf); LSE = np.zeros((T, hq))
    dQ = np.zeros_like(qf); dK = np.zeros_like(kf); dV = np.zeros_like(vf)
    for n in range(len(cu) - 1):
        a, b = cu[n], cu[n + 1]
        L = b - a
        tril = np.tril(np.ones((L, L), bool))
        for h in range(hq):
            g = h // G
            S = scale * qf[a:b, h] @ kf[a:b, g].T
            E = np.where(tril, np.exp(S), 0.0)
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


@pytest.mark.parametrize("hq,hkv,D", [(4, 4, 8), (6, 2, 16), (5, 1, 8)])
def test_dense_matrix_small(hq, hkv, D):
    rng = np.random.default_rng(1)
    lens = [1, 7, 32, 13]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(cu[-1])
    q, do = _rand_bits(rng, (T, hq, D)), _rand_bits(rng, (T, hq, D))
    k, v = _rand_bits(rng, (T, hkv, D)), _rand_bits(rng, (T, hkv, D))
    scale = 1.0 / np.sqrt(D)
    O, LSE = oattn.attn_fwd(q, k, v, cu, scale)
    dQ, dK, dV = oattn.attn_bwd(q, k, v, do, cu, scale)
    rO, rLSE, rdQ, rdK, rdV = _dense_reference(q, k, v, do, cu, scale)
    for got, ref in ((O, rO), (LSE, rLSE), (dQ, rdQ), (dK, rdK), (dV, rdV)):
        np.testing.assert_allclose(got, ref, rtol=1e-11, atol=1e-12)


def test_single_token_sequence():
    """L = 1: O = V_0 and LSE = scale * q_0 . k_0 (softmax over one key)."""
    rng = np.random.default_rng(2)
    q, k, v = _rand_bits(rng, (1, 2, 8)), _rand_bits(rng, (1, 1, 8)), _rand_bits(rng, (1, 1, 8))
    O, LSE = oattn.attn_fwd(q, k, v, np.array([0, 1], np.int32), 0.3)
    qf, kf, vf = (synth.bf16_bits_to_f64(x) for x in (q, k, v))
    np.testing.assert_allclose(O[0, 0], vf[0, 0], rtol=0, atol=1e-15)
    np.testing.assert_allclose(O[0, 1], vf[0, 0], rtol=0, atol=1e-15)
    np.testing.assert_allclose(LSE[0], 0.3 * (qf[0] @ kf[0, 0]), rtol=1e-14)


def test_constant_keys_closed_form():
    """All keys equal: softmax is uniform over the i+1 visible keys, so
    LSE_i = scale q_i.k + ln(i+1) and O_i = mean(V_0..V_i).  A wrong mask direction,
    an off-by-one in the causal range or a missing scale shows here."""
    rng = np.random.default_rng(3)
    L, hq, hkv, D = 40, 4, 2, 16
    q, v = _rand_bits(rng, (L, hq, D)), _rand_bits(rng, (L, hkv, D))
    k1 = _rand_bits(rng, (1, hkv, D))
    k = np.repeat(k1, L, axis=0)
    scale = 0.25
    O, LSE = oattn.attn_fwd(q, k, v, np.array([0, L], np.int32), scale)
    qf, kf, vf = (synth.bf16_bits_to_f64(x) for x in (q, k1, v))
    prefix_mean = np.cumsum(vf, axis=0) / np.arange(1, L + 1)[:, None, None]
    for h in range(hq):
        g = h // (hq // hkv)
        np.testing.assert_allclose(LSE[:, h], scale * qf[:, h] @ kf[0, g] + np.log(np.arange(1, L + 1)),
                                   rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(O[:, h], prefix_mean[:, g], rtol=1e-13, atol=1e-14)


def test_constant_values_zero_dq_dk():
    """V constant over keys: O equals that constant for every row, and the loss sum(O*dO)
    no longer depends on Q or K, so dQ = dK = 0; dV_j = sum_i p_ij dO_i still sums to
    sum_i dO_i over the keys."""
    rng = np.random.default_rng(4)
    L, hq, hkv, D = 24, 4, 2, 8
    q, k, do = _rand_bits(rng, (L, hq, D)), _rand_bits(rng, (L, hkv, D)), _rand_bits(rng, (L, hq, D))
    v = np.repeat(_rand_bits(rng, (1, hkv, D)), L, axis=0)
    cu = np.array([0, L], np.int32)
    O, _ = oattn.attn_fwd(q, k, v, cu, 0.4)
    vf, dof = synth.bf16_bits_to_f64(v), synth.bf16_bits_to_f64(do)
    for h in range(hq):
        np.testing.assert_allclose(O[:, h], np.broadcast_to(vf[0, h // 2], (L, D)), rtol=1e-14, atol=1e-15)
    dQ, dK, dV = oattn.attn_bwd(q, k, v, do, cu, 0.4)
    assert np.abs(dQ).max() < 1e-13 and np.abs(dK).max() < 1e-13
    for g in range(hkv):
        np.testing.assert_allclose(dV[:, g].sum(0), dof[:, 2 * g:2 * g + 2].sum((0, 1)), rtol=1e-12)


def test_row_sum_invariants_packed():
    """Two identities that hold for every packed sequence and KV head:
    (1) sum_j p_ij = 1, so sum_j dV_j equals the sum of dO over the sequence's rows and the
        group's query heads;
    (2) adding one constant vector to every key of a sequence shifts all visible scores of a
        row equally, which softmax ignores, so the loss is invariant and sum_j dK_j = 0."""
    rng = np.random.default_rng(5)
    lens = [9, 30, 5]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T, hq, hkv, D = int(cu[-1]), 6, 3, 8
    q, do = _rand_bits(rng, (T, hq, D)), _rand_bits(rng, (T, hq, D))
    k, v = _rand_bits(rng, (T, hkv, D)), _rand_bits(rng, (T, hkv, D))
    dQ, dK, dV = oattn.attn_bwd(q, k, v, do, cu, 0.35)
    dof = synth.bf16_bits_to_f64(do)
    for n in range(3):
        a, b = cu[n], cu[n + 1]
        for g in range(hkv):
            np.testing.assert_allclose(dV[a:b, g].sum(0), dof[a:b, 2 * g:2 * g + 2].sum((0, 1)), rtol=1e-11, atol=1e-12)
            assert np.abs(dK[a:b, g].sum(0)).max() < 1e-11


def test_torch_sdpa_float64_special_case():
    """Library routine on the special case it covers: one unsharded sequence,
    torch CPU float64 scaled_dot_product_attention(is_causal=True) with autograd;
    grouped heads expressed with repeat_interleave."""
    rng = np.random.default_rng(6)
    L, hq, hkv, D = 48, 8, 2, 16
    q, do = _rand_bits(rng, (L, hq, D)), _rand_bits(rng, (L, hq, D))
    k, v = _rand_bits(rng, (L, hkv, D)), _rand_bits(rng, (L, hkv, D))
    scale = 1.0 / np.sqrt(D)
    cu = np.array([0, L], np.int32)
    O, LSE = oattn.attn_fwd(q, k, v, cu, scale)
    dQ, dK, dV = oattn.attn_bwd(q, k, v, do, cu, scale)

    tq = torch.tensor(synth.bf16_bits_to_f64(q), requires_grad=True)
    tk = torch.tensor(synth.bf16_bits_to_f64(k), requires_grad=True)
    tv = torch.tensor(synth.bf16_bits_to_f64(v), requires_grad=True)
    tdo = torch.tensor(synth.bf16_bits_to_f64(do))
    G = hq // hkv
    kx = tk.repeat_interleave(G, dim=1)
    vx = tv.repeat_interleave(G, dim=1)
    out = torch.nn.functional.scaled_dot_product_attention(
        tq.permute(1, 0, 2)[None], kx.permute(1, 0, 2)[None], vx.permute(1, 0, 2)[None],
        is_causal=True, scale=scale)[0].permute(1, 0, 2)
    (out * tdo).sum().backward()
    np.testing.assert_allclose(O, out.detach().numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dQ, tq.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(dK, tk.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(dV, tv.grad.numpy(), rtol=1e-9, atol=1e-11)
    # LSE against torch.logsumexp of the masked scaled scores
    S = scale * torch.einsum("ihc,jhc->hij", tq.detach(), kx.detach())
    S = S.masked_fill(~torch.tril(torch.ones(L, L, dtype=torch.bool)), float("-inf"))
    np.testing.assert_allclose(LSE, torch.logsumexp(S, dim=2).T.numpy(), rtol=1e-12, atol=1e-12)


def test_finite_differences():
    """Central differences of loss = sum(O*dO) in fp64 on values that are exactly
    representable in bf16 (so the perturbed point is evaluated by a float path here)."""
    rng = np.random.default_rng(7)
    lens = [5, 11]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T, hq, hkv, D = 16, 2, 1, 4
    q, do = _rand_bits(rng, (T, hq, D)), _rand_bits(rng, (T, hq, D))
    k, v = _rand_bits(rng, (T, hkv, D)), _rand_bits(rng, (T, hkv, D))
    scale = 0.5
    dQ, dK, dV = oattn.attn_bwd(q, k, v, do, cu, scale)
    qf, kf, vf, dof = (synth.bf16_bits_to_f64(x) for x in (q, k, v, do))

    def loss(qx, kx, vx):
        tot = 0.0
        for n in range(2):
            a, b = cu[n], cu[n + 1]
            for h in range(hq):
                for i in range(a, b):
                    s = scale * kx[a:i + 1, 0] @ qx[i, h]
                    p = np.exp(s - s.max()); p /= p.sum()
                    tot += (p @ vx[a:i + 1, 0]) @ dof[i, h]
        return tot

    eps = 1e-5
    for name, arr, grad in (("q", qf, dQ), ("k", kf, dK), ("v", vf, dV)):
        for idx in [(0, 0, 0), (3, 0, 1), (7, 0, 2), (15, 0, 3), (9, 0, 0)] + ([(6, 1, 2)] if name == "q" else []):
            ap, am = arr.copy(), arr.copy()
            ap[idx] += eps; am[idx] -= eps
            args_p = {"q": (ap, kf, vf), "k": (qf, ap, vf), "v": (qf, kf, ap)}[name]
            args_m = {"q": (am, kf, vf), "k": (qf, am, vf), "v": (qf, kf, am)}[name]
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(fd - grad[idx]) < 1e-7 * max(1.0, abs(fd)), (name, idx, fd, grad[idx])


def test_row_subset_and_rank_partial_sum():
    """Rows are independent: asking for a subset gives the same rows; dK/dV restricted to
    disjoint row subsets add up to the full dK/dV."""
    rng = np.random.default_rng(8)
    lens = [20, 12]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T, hq, hkv, D = 32, 4, 2, 8
    q, do = _rand_bits(rng, (T, hq, D)), _rand_bits(rng, (T, hq, D))
    k, v = _rand_bits(rng, (T, hkv, D)), _rand_bits(rng, (T, hkv, D))
    O, LSE = oattn.attn_fwd(q, k, v, cu, 0.3)
    dQ, dK, dV = oattn.attn_bwd(q, k, v, do, cu, 0.3)
    perm = rng.permutation(T)
    A, B = np.sort(perm[:13]), np.sort(perm[13:])
    OA, LA = oattn.attn_fwd(q, k, v, cu, 0.3, rows=A)
    np.testing.assert_array_equal(OA, O[A]); np.testing.assert_array_equal(LA, LSE[A])
    dQA, dKA, dVA = oattn.attn_bwd(q, k, v, do, cu, 0.3, rows=A)
    dQB, dKB, dVB = oattn.attn_bwd(q, k, v, do, cu, 0.3, rows=B)
    np.testing.assert_array_equal(dQA, dQ[A])
    np.testing.assert_allclose(dKA + dKB, dK, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dVA + dVB, dV, rtol=1e-12, atol=1e-13)
    # a key subset is the same rows of the full result
    keys = np.array([31, 0, 7, 19], np.int64)
    dKs, dVs = oattn.attn_dkv(q, k, v, do, cu, 0.3, A, OA, LA, keys=keys)
    np.testing.assert_array_equal(dKs, dKA[keys]); np.testing.assert_array_equal(dVs, dVA[keys])


def test_bf16_roundtrip_and_rne():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0, 3.0e38], np.float32)
    b = synth.f32_to_bf16_bits(x)
    # 1 + 2^-8 is a tie between 1.0 (even mantissa) and 1 + 2^-7: rounds to even = 1.0
    assert b[1] == 0x3F80
    # 1 + 3*2^-8 is a tie between mantissa 1 and 2: rounds to even = 2 -> 1 + 2^-6
    assert b[2] == 0x3F82
    t = torch.tensor(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(b, t)
    r = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    np.testing.assert_array_equal(synth.f32_to_bf16_bits(r),
                                  torch.tensor(r).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
    np.testing.assert_array_equal(synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(r)),
                                  torch.tensor(r).to(torch.bfloat16).float().numpy())
