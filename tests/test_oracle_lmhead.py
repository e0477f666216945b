"""Pins for the oracle's LM head / confidence (CPU only)."""
import math

import numpy as np
import pytest

import oracle
from paper_2604_04215_amd import synth
from brute_force import lmhead_brute


def rnd(seed, shape, std=1.0):
    return synth.normal_bf16(4321, 55, (seed,), shape, std)


def f64(u):
    return synth.bf16_bits_to_f64(u)


def bits(x):
    return synth.f32_to_bf16_bits(np.asarray(x, np.float32))


@pytest.mark.parametrize("forbid,inv_t", [(-1, 1.0), (5, 1.0), (-1, 0.5), (0, 2.0)])
def test_brute_force_tiny(forbid, inv_t):
    M, Dh, V = 5, 12, 37
    h, w = rnd(1, (M, Dh)), rnd(2, (V, Dh), 0.7)
    r = oracle.lmhead(h, w, forbid_token=forbid, inv_temperature=inv_t)
    for i in range(M):
        conf, tok, lse, zmax, z2 = lmhead_brute(f64(h)[i].tolist(), f64(w).tolist(), inv_t, forbid)
        assert r["tok"][i] == tok
        assert abs(r["conf"][i] - conf) < 1e-13
        assert abs(r["lse"][i] - lse) < 1e-12 and abs(r["zmax"][i] - zmax) < 1e-12
        assert abs(r["z2nd"][i] - z2) < 1e-12
    if forbid >= 0:
        assert np.all(r["tok"] != forbid)


def test_closed_form_single_spike_and_threshold_boundary():
    # z = (a, 0, ..., 0): conf = e^a / (e^a + V - 1)
    Dh, V = 8, 64
    h = bits(np.eye(1, Dh, 0))                      # h = e_0
    for a in (0.5, 2.0, 8.0):
        wf = np.zeros((V, Dh), np.float32)
        wf[3, 0] = a
        r = oracle.lmhead(h, bits(wf))
        assert r["tok"][0] == 3
        assert abs(r["conf"][0] - math.exp(a) / (math.exp(a) + V - 1)) < 1e-14
        assert abs(r["zmax"][0] - a) < 1e-15 and r["z2nd"][0] == 0.0
    # a = ln(9 (V-1)) puts the confidence at 0.9: check on the bf16-rounded a actually stored
    a = float(f64(bits([math.log(9 * (V - 1))]))[0])
    wf = np.zeros((V, Dh), np.float32)
    wf[10, 0] = a
    r = oracle.lmhead(h, bits(wf))
    assert abs(r["conf"][0] - 1.0 / (1.0 + (V - 1) * math.exp(-a))) < 1e-14
    assert abs(r["conf"][0] - 0.9) < 2e-3


def test_all_equal_logits_lowest_index_and_uniform_conf():
    Dh, V = 8, 50
    h = bits(np.ones((2, Dh)))
    w = bits(np.full((V, Dh), 0.25))
    r = oracle.lmhead(h, w)
    assert np.all(r["tok"] == 0)
    assert np.allclose(r["conf"], 1.0 / V, atol=1e-15)
    assert np.allclose(r["z2nd"], r["zmax"])                    # a tie: runner-up equals the max
    r2 = oracle.lmhead(h, w, forbid_token=0)
    assert np.all(r2["tok"] == 1) and np.allclose(r2["conf"], 1.0 / (V - 1), atol=1e-15)


def test_identity_block_picks_argmax_of_hidden():
    Dh = 16
    h = rnd(3, (6, Dh))
    w = bits(np.eye(Dh) * 2.0)                                   # z = 2 h
    r = oracle.lmhead(h, w)
    hf = f64(h)
    assert np.array_equal(r["tok"], hf.argmax(axis=1).astype(np.int32))
    assert np.allclose(r["zmax"], 2.0 * hf.max(axis=1))
    # transposed operand would index hidden by vocab: a non-square W catches shape slips
    w2 = bits(np.eye(Dh + 3, Dh))
    r2 = oracle.lmhead(h, w2)
    assert np.array_equal(r2["tok"], np.where(hf.max(axis=1) > 0, hf.argmax(axis=1), Dh).astype(np.int32))


def test_invariants_and_library_cross_check():
    from scipy.special import logsumexp
    M, Dh, V = 7, 32, 211
    h, w = rnd(4, (M, Dh)), rnd(5, (V, Dh), 0.8)
    r = oracle.lmhead(h, w)
    z = f64(h) @ f64(w).T
    assert np.allclose(r["lse"], logsumexp(z, axis=1), atol=1e-12)
    assert np.array_equal(r["tok"], z.argmax(axis=1))
    assert np.allclose(np.exp(z - r["lse"][:, None]).sum(axis=1), 1.0, atol=1e-13)
    assert np.all(r["conf"] <= 1.0) and np.all(r["conf"] >= 1.0 / V)
    part = np.partition(z, V - 2, axis=1)
    assert np.allclose(r["z2nd"], part[:, V - 2], atol=1e-12)
    # temperature: lse(z * c) of the scaled logits
    r2 = oracle.lmhead(h, w, inv_temperature=0.25)
    assert np.allclose(r2["lse"], logsumexp(z * 0.25, axis=1), atol=1e-12)
    # merging (m, s, idx, m2) of two vocab halves reproduces the whole
    a, b = oracle.lmhead(h, w[:100]), oracle.lmhead(h, w[100:])
    m = np.maximum(a["zmax"], b["zmax"])
    s = np.exp(a["lse"] - m) + np.exp(b["lse"] - m)
    assert np.allclose(m + np.log(s), r["lse"], atol=1e-12)
    tok = np.where(a["zmax"] >= b["zmax"], a["tok"], b["tok"] + 100)
    assert np.array_equal(tok, r["tok"])
    z2 = np.maximum(np.maximum(a["z2nd"], b["z2nd"]), np.minimum(a["zmax"], b["zmax"]))
    assert np.allclose(z2, r["z2nd"], atol=1e-12)


def test_row_gather_and_target_logit():
    R, Dh, V = 9, 16, 40
    h, w = rnd(6, (R, Dh)), rnd(7, (V, Dh))
    full = oracle.lmhead(h, w)
    idx = np.array([7, 2, 2, 8], np.int32)
    tgt = np.array([0, 39, 5, 17], np.int32)
    sub = oracle.lmhead(h, w, row_idx=idx, target=tgt)
    for key in ("conf", "tok", "lse", "zmax", "z2nd"):
        assert np.array_equal(sub[key], full[key][idx])
    z = f64(h) @ f64(w).T
    assert np.allclose(sub["zt"], z[idx, tgt], atol=1e-12)
    # log p(target) = z_target - lse, and the arg-max token's log-prob is log(conf)
    sub2 = oracle.lmhead(h, w, row_idx=idx, target=full["tok"][idx])
    assert np.allclose(sub2["zt"] - sub2["lse"], np.log(sub2["conf"]), atol=1e-12)
    empty = oracle.lmhead(h, w, row_idx=np.zeros(0, np.int32))
    assert empty["conf"].shape == (0,)


def test_margin_and_negative_entropy_scores():
    import scipy.stats
    M, Dh, V = 6, 16, 23
    h, w = rnd(31, (M, Dh)), rnd(32, (V, Dh), 0.6)
    r = oracle.lmhead(h, w, forbid_token=4)
    z = f64(h) @ f64(w).T
    z[:, 4] = -np.inf
    p = np.exp(z - z.max(1, keepdims=True))
    p /= p.sum(1, keepdims=True)
    top2 = np.sort(p, axis=1)[:, -2:]
    assert np.allclose(r["margin"], top2[:, 1] - top2[:, 0], atol=1e-13)
    assert np.allclose(r["neg_entropy"], -scipy.stats.entropy(p, axis=1), atol=1e-12)     # library routine
    # closed forms: uniform logits -> -log V (one token forbidden: -log(V - 1)), margin 0
    h0 = np.zeros((2, Dh), np.uint16)
    u = oracle.lmhead(h0, w)
    assert np.allclose(u["neg_entropy"], -math.log(V), atol=1e-13) and np.allclose(u["margin"], 0, atol=1e-15)
    u = oracle.lmhead(h0, w, forbid_token=0)
    assert np.allclose(u["neg_entropy"], -math.log(V - 1), atol=1e-13)
    # z = (a, b, 0, ..., 0): margin = (e^a - e^b) / Z, entropy from the three distinct probabilities
    a, b, Vs = 3.0, 1.5, 40
    wf = np.zeros((Vs, Dh), np.float32)
    wf[7, 0], wf[20, 0] = a, b
    s = oracle.lmhead(bits(np.eye(1, Dh, dtype=np.float32)), bits(wf))
    Z = math.exp(a) + math.exp(b) + Vs - 2
    pa, pb, p0 = math.exp(a) / Z, math.exp(b) / Z, 1 / Z
    assert abs(s["margin"][0] - (pa - pb)) < 1e-14
    assert abs(s["neg_entropy"][0] - (pa * math.log(pa) + pb * math.log(pb) + (Vs - 2) * p0 * math.log(p0))) < 1e-13
    # a sharper distribution (lower temperature) has higher negative entropy
    cold = oracle.lmhead(h, w, inv_temperature=3.0)
    warm = oracle.lmhead(h, w, inv_temperature=0.3)
    assert np.all(cold["neg_entropy"] > warm["neg_entropy"]) and np.all(cold["neg_entropy"] <= 1e-15)
