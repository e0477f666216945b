"""Pins for the oracle's attention gradient (CPU only): automatic differentiation of a plain float64 softmax
attention (library routine), central finite differences of the pinned forward oracle's own definition, and
structural identities (rows of dS sum to zero; a hidden key gets no gradient)."""
import numpy as np
import pytest
import torch

import oracle
from oracle import KV
from oracle import backward as obw
from paper_2604_04215_amd import synth


def rnd(seed, shape):
    return synth.normal_bf16(606, 9, (seed,), shape)


def f64(u):
    return synth.bf16_bits_to_f64(u)


def torch_reference(q, segs, d_out, vis, scale):
    """autograd through softmax(scale QK^T + mask) V in float64, GQA by repeating KV heads"""
    Q = torch.tensor(f64(q), requires_grad=True)
    Ks = [torch.tensor(f64(s.k), requires_grad=True) for s in segs]
    Vs = [torch.tensor(f64(s.v), requires_grad=True) for s in segs]
    K, V = torch.cat(Ks, dim=2), torch.cat(Vs, dim=2)
    g = Q.shape[2] // K.shape[1]
    Kr, Vr = K.repeat_interleave(g, dim=1), V.repeat_interleave(g, dim=1)          # [B, Hq, Lk, d]
    s = scale * torch.einsum("bihc,bhjc->bhij", Q, Kr)
    s = s.masked_fill(~torch.tensor(vis)[None, None], float("-inf"))
    P = torch.softmax(s, dim=-1)
    P = torch.nan_to_num(P, nan=0.0)                                               # rows that see nothing
    O = torch.einsum("bhij,bhjc->bihc", P, Vr)
    (O * torch.tensor(f64(d_out))).sum().backward()
    return Q.grad.numpy(), [(k.grad.numpy(), v.grad.numpy()) for k, v in zip(Ks, Vs)]


CASES = [
    dict(mode="full", bs=0, q_pos0=0, rules=("causal", "causal")),
    dict(mode="block_causal", bs=4, q_pos0=8, rules=("causal", "causal")),
    dict(mode="block_causal", bs=4, q_pos0=0, rules=("earlier", "same")),
    dict(mode="block_causal", bs=3, q_pos0=0, rules=("same", "earlier")),
]


@pytest.mark.parametrize("case", CASES)
def test_against_autograd(case):
    B, Lq, Hq, Hkv, d, L0, L1 = 2, 12, 4, 2, 8, 12, 12
    q, dO = rnd(1, (B, Lq, Hq, d)), rnd(2, (B, Lq, Hq, d))
    segs = [KV(rnd(3, (B, Hkv, L0, d)), rnd(4, (B, Hkv, L0, d)), 0, case["rules"][0]),
            KV(rnd(5, (B, Hkv, L1, d)), rnd(6, (B, Hkv, L1, d)), 0 if case["rules"][0] != "causal" else L0, case["rules"][1])]
    dQ, dKV = obw.attention_backward(q, segs, dO, mask_mode=case["mode"], bs=case["bs"], q_pos0=case["q_pos0"])
    vis = obw.visibility(Lq, segs, mask_mode=case["mode"], bs=case["bs"], q_pos0=case["q_pos0"])
    rQ, rKV = torch_reference(q, segs, dO, vis, 1.0 / np.sqrt(d))
    assert np.allclose(dQ, rQ, atol=1e-12)
    for (dk, dv), (rk, rv) in zip(dKV, rKV):
        assert np.allclose(dk, rk, atol=1e-12) and np.allclose(dv, rv, atol=1e-12)
    # the visibility used here is the forward oracle's: masked forward outputs agree with the dense softmax
    O, _ = oracle.attention(q, segs, mask_mode=case["mode"], bs=case["bs"], q_pos0=case["q_pos0"])
    K, V = np.concatenate([f64(s.k) for s in segs], 2), np.concatenate([f64(s.v) for s in segs], 2)
    for h in range(Hq):
        s = np.where(vis, (f64(q)[0, :, h] @ K[0, h // 2].T) / np.sqrt(d), -np.inf)
        with np.errstate(invalid="ignore"):
            P = np.nan_to_num(np.exp(s - s.max(1, keepdims=True)) / np.exp(s - s.max(1, keepdims=True)).sum(1, keepdims=True))
        assert np.allclose(O[0, :, h], P @ V[0, h // 2], atol=1e-12)


def test_finite_differences_of_the_scalar_loss():
    # L(Q, K, V) = sum(O * dO); perturb single entries (values that stay exact in bf16: +- 2^-6 on small integers)
    B, Lq, Hq, Hkv, d, Lk = 1, 5, 2, 1, 4, 7
    g = np.random.default_rng(0)
    mk = lambda *s: synth.f32_to_bf16_bits(g.integers(-3, 4, s).astype(np.float32) / 2)
    q, k, v, dO = mk(B, Lq, Hq, d), mk(B, Hkv, Lk, d), mk(B, Hkv, Lk, d), mk(B, Lq, Hq, d)
    dQ, [(dK, dV)] = obw.attention_backward(q, [KV(k, v, 0)], dO, mask_mode="block_causal", bs=2, q_pos0=2)

    def loss(q_, k_, v_):
        O, _ = oracle.attention(q_, [KV(k_, v_, 0)], mask_mode="block_causal", bs=2, q_pos0=2)
        return float((O * f64(dO)).sum())

    eps = 2.0 ** -6
    for name, arr, grad, idxs in (("q", q, dQ, [(0, 0, 0, 0), (0, 4, 1, 3), (0, 2, 1, 1)]),
                                  ("k", k, dK, [(0, 0, 0, 0), (0, 0, 5, 2), (0, 0, 6, 3)]),
                                  ("v", v, dV, [(0, 0, 1, 1), (0, 0, 6, 0)])):
        for idx in idxs:
            vals = []
            for sgn in (+1, -1):
                a = f64(arr).astype(np.float32)
                a[idx] += sgn * eps
                bits = synth.f32_to_bf16_bits(a)
                assert synth.bf16_bits_to_f64(bits)[idx] == float(a[idx])          # still exact
                args = dict(q=q, k=k, v=v)
                args[name] = bits
                vals.append(loss(args["q"], args["k"], args["v"]))
            fd = (vals[0] - vals[1]) / (2 * eps)
            assert abs(fd - grad[idx]) < 2e-4 * max(1.0, abs(fd)), (name, idx, fd, grad[idx])


def test_structure():
    B, Lq, Hq, Hkv, d, Lk, bs = 1, 8, 2, 2, 8, 16, 4
    q, dO, k, v = rnd(11, (B, Lq, Hq, d)), rnd(12, (B, Lq, Hq, d)), rnd(13, (B, Hkv, Lk, d)), rnd(14, (B, Hkv, Lk, d))
    v = synth.f32_to_bf16_bits((np.round(f64(v) * 8) / 8).astype(np.float32))     # eighths: v + 1 stays exact in bf16
    dQ, [(dK, dV)] = obw.attention_backward(q, [KV(k, v, 0)], dO, mask_mode="block_causal", bs=bs, q_pos0=0)
    # keys beyond the last query block are invisible to everyone: no gradient reaches them
    assert not dK[:, :, Lq:].any() and not dV[:, :, Lq:].any() and dK[:, :, :Lq].any()
    # adding a constant vector to every V row shifts O by that constant and leaves dQ, dK unchanged
    v2 = synth.f32_to_bf16_bits((f64(v) + 1.0).astype(np.float32))
    assert np.array_equal(synth.bf16_bits_to_f64(v2), f64(v) + 1.0)
    dQ2, [(dK2, _)] = obw.attention_backward(q, [KV(k, v2, 0)], dO, mask_mode="block_causal", bs=bs, q_pos0=0)
    assert np.allclose(dQ, dQ2, atol=1e-10) and np.allclose(dK, dK2, atol=1e-10)
    # dV rows sum to the sum of dO rows (every query's probabilities sum to one)
    assert np.allclose(dV.sum(axis=2), f64(dO).sum(axis=1), atol=1e-12)
