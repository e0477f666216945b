"""Pins for the oracle's packed variable-length attention (CPU only).

The packed form is pinned against formulations that never slice the buffer by sequence: a dense
[T, T] same-sequence visibility matrix fed to a library softmax, a pure-Python brute force on the
padded batch, and isolation / permutation identities.  A wrong offset, an off-by-one sequence end,
a mixed-up LSE layout or leakage between neighbours fails at least one of them."""
import numpy as np
import pytest
import scipy.special

import oracle
from paper_2604_04215_amd import synth
from brute_force import attention_brute


def rnd(seed, shape):
    return synth.normal_bf16(4242, 13, (seed,), shape)


def f64(u):
    return synth.bf16_bits_to_f64(u)


def packed(lens, Hq, Hkv, d, seed=0):
    T = int(np.sum(lens))
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    return rnd(seed + 1, (T, Hq, d)), rnd(seed + 2, (T, Hkv, d)), rnd(seed + 3, (T, Hkv, d)), cu


@pytest.mark.parametrize("mode,bs", [("full", 0), ("block_causal", 4)])
def test_dense_same_sequence_mask_with_library_softmax(mode, bs):
    lens = [5, 1, 0, 9, 3]
    Hq, Hkv, d = 4, 2, 8
    q, k, v, cu = packed(lens, Hq, Hkv, d)
    O, lse = oracle.attention_varlen(q, k, v, cu, mask_mode=mode, bs=bs)
    T = q.shape[0]
    seq_of = np.repeat(np.arange(len(lens)), lens)
    pos = np.arange(T) - cu[:-1][seq_of]
    vis = seq_of[:, None] == seq_of[None, :]
    if mode == "block_causal":
        vis &= (pos[None, :] // bs) <= (pos[:, None] // bs)
    Q, K, V = f64(q), f64(k), f64(v)
    g = Hq // Hkv
    for h in range(Hq):
        s = (Q[:, h] @ K[:, h // g].T) / np.sqrt(d)
        s = np.where(vis, s, -np.inf)
        p = scipy.special.softmax(s, axis=1)
        assert np.allclose(O[:, h], p @ V[:, h // g], atol=1e-12)
        assert np.allclose(lse[h], scipy.special.logsumexp(s, axis=1), atol=1e-12)


def test_pure_python_brute_force_on_padded_batch():
    lens = [3, 6, 2]
    Hq, Hkv, d = 2, 1, 4
    q, k, v, cu = packed(lens, Hq, Hkv, d, seed=10)
    O, lse = oracle.attention_varlen(q, k, v, cu)
    Lmax = max(lens)
    B = len(lens)
    qp = np.zeros((B, Lmax, Hq, d)); kp = np.zeros((B, Hkv, Lmax, d)); vp = np.zeros((B, Hkv, Lmax, d))
    key_ok = [[0] * Lmax for _ in range(B)]
    for b, n in enumerate(lens):
        qp[b, :n] = f64(q)[cu[b]:cu[b + 1]]
        kp[b, :, :n] = f64(k)[cu[b]:cu[b + 1]].transpose(1, 0, 2)
        vp[b, :, :n] = f64(v)[cu[b]:cu[b + 1]].transpose(1, 0, 2)
        key_ok[b][:n] = [1] * n
    Ob, lb = attention_brute(qp.tolist(), kp.tolist(), vp.tolist(), list(range(Lmax)), 0, "full", 0, key_ok=key_ok)
    Ob, lb = np.array(Ob), np.array(lb)
    for b, n in enumerate(lens):
        assert np.allclose(O[cu[b]:cu[b + 1]], Ob[b, :n], atol=1e-12)
        assert np.allclose(lse[:, cu[b]:cu[b + 1]], lb[b, :, :n], atol=1e-12)


def test_isolation_and_order_of_sequences():
    lens = [7, 4, 6]
    Hq, Hkv, d = 4, 4, 8
    q, k, v, cu = packed(lens, Hq, Hkv, d, seed=20)
    O, lse = oracle.attention_varlen(q, k, v, cu)
    # changing every token of the middle sequence leaves its neighbours untouched
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    sl = slice(cu[1], cu[2])
    q2[sl], k2[sl], v2[sl] = rnd(31, q[sl].shape), rnd(32, k[sl].shape), rnd(33, v[sl].shape)
    O2, lse2 = oracle.attention_varlen(q2, k2, v2, cu)
    keep = np.r_[0:cu[1], cu[2]:cu[3]]
    assert np.array_equal(O[keep], O2[keep]) and np.array_equal(lse[:, keep], lse2[:, keep])
    assert not np.allclose(O[sl], O2[sl])
    # packing the sequences in another order permutes the result the same way
    order = [2, 0, 1]
    idx = np.concatenate([np.arange(cu[b], cu[b + 1]) for b in order])
    cu3 = np.concatenate([[0], np.cumsum([lens[b] for b in order])])
    O3, lse3 = oracle.attention_varlen(q[idx], k[idx], v[idx], cu3)
    assert np.allclose(O3, O[idx], atol=1e-14) and np.allclose(lse3, lse[:, idx], atol=1e-14)


def test_single_token_sequences_return_their_own_value():
    # a sequence of one token: softmax over one key is 1, so O = V (per GQA group) and LSE = scale * q.k
    Hq, Hkv, d = 4, 2, 16
    q, k, v, cu = packed([1, 1, 1], Hq, Hkv, d, seed=40)
    O, lse = oracle.attention_varlen(q, k, v, cu)
    for h in range(Hq):
        assert np.allclose(O[:, h], f64(v)[:, h // 2], atol=1e-15)
        assert np.allclose(lse[h], (f64(q)[:, h] * f64(k)[:, h // 2]).sum(-1) / 4.0, atol=1e-13)


def test_synthetic_recipe_shapes():
    cfg = synth.VARLEN["miniv1"]
    q, k, v, cu = synth.varlen_qkv(cfg)
    lens = np.diff(cu)
    assert cu[0] == 0 and len(cu) == cfg.B + 1 and q.shape == (cu[-1], cfg.Hq, cfg.d)
    assert lens.min() >= cfg.prompt_lo + cfg.resp_lo and lens.max() <= cfg.max_len
    q2, _, _, cu2 = synth.varlen_qkv(cfg)
    assert np.array_equal(q, q2) and np.array_equal(cu, cu2)
