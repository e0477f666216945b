"""Pins for the oracle's per-sequence masked log-likelihood (the sum that Eq. 2 / Eq. 3 weight by 1/t). CPU only."""
import math

import numpy as np
import scipy.special

import oracle
from paper_2604_04215_amd import synth


def rnd(seed, shape, std=1.0):
    return synth.normal_bf16(977, 3, (seed,), shape, std)


def f64(u):
    return synth.bf16_bits_to_f64(u)


def test_uniform_logits_closed_form():
    # zero hidden states: every token has probability 1/V (1/(V-1) with one token forbidden)
    B, n, Dh, V = 3, 7, 16, 41
    h = np.zeros((B, n, Dh), np.uint16)
    w = rnd(1, (V, Dh))
    tgt = np.arange(B * n).reshape(B, n) % (V - 1)
    mask = np.zeros((B, n), np.uint8)
    mask[0, :] = 1
    mask[1, [2, 5]] = 1
    out, cnt = oracle.seq_logprob(h, w, tgt, mask)
    assert cnt.tolist() == [7, 2, 0]
    assert np.allclose(out, [-7 * math.log(V), -2 * math.log(V), 0.0], atol=1e-12)
    out2, _ = oracle.seq_logprob(h, w, tgt, mask, forbid_token=V - 1, weight=[-0.5, 2.0, 3.0])
    assert np.allclose(out2, [3.5 * math.log(V - 1), -4 * math.log(V - 1), 0.0], atol=1e-12)


def test_pure_python_brute_force():
    B, n, Dh, V = 2, 5, 6, 11
    h, w = rnd(2, (B, n, Dh)), rnd(3, (V, Dh), 0.8)
    tgt = (np.arange(B * n).reshape(B, n) * 7 + 3) % V
    mask = np.array([[1, 0, 1, 1, 0], [0, 0, 0, 1, 1]], np.uint8)
    out, cnt = oracle.seq_logprob(h, w, tgt, mask)
    H, W = f64(h).tolist(), f64(w).tolist()
    for b in range(B):
        tot, c = 0.0, 0
        for i in range(n):
            if not mask[b, i]:
                continue
            z = [sum(H[b][i][d] * W[v][d] for d in range(Dh)) for v in range(V)]
            tot += z[tgt[b, i]] - math.log(sum(math.exp(x) for x in z))
            c += 1
        assert c == cnt[b] and abs(tot - out[b]) < 1e-12


def test_library_log_softmax_and_normalisation():
    B, n, Dh, V = 2, 9, 32, 53
    h, w = rnd(4, (B, n, Dh)), rnd(5, (V, Dh), 0.5)
    mask = (np.arange(B * n).reshape(B, n) % 3 != 1).astype(np.uint8)
    logp = scipy.special.log_softmax(f64(h) @ f64(w).T, axis=-1)          # [B, n, V]
    tgt = (np.arange(B * n).reshape(B, n) * 5) % V
    out, _ = oracle.seq_logprob(h, w, tgt, mask)
    want = (np.take_along_axis(logp, tgt[..., None], -1)[..., 0] * mask).sum(1)
    assert np.allclose(out, want, atol=1e-11)
    # one masked position: exp of the result over every possible target sums to one
    one = np.zeros((B, n), np.uint8)
    one[:, 4] = 1
    tot = np.zeros(B)
    for v in range(V):
        o, _ = oracle.seq_logprob(h, w, np.full((B, n), v), one)
        tot += np.exp(o)
    assert np.allclose(tot, 1.0, atol=1e-12)


def test_additivity_over_mask_split():
    # a sum over a mask is the sum over any partition of it; a transposed target/mask index would break this
    B, n, Dh, V = 3, 8, 16, 29
    h, w = rnd(6, (B, n, Dh)), rnd(7, (V, Dh))
    tgt = (np.arange(B * n).reshape(B, n) * 11 + 1) % V
    m = np.ones((B, n), np.uint8)
    a = m.copy(); a[:, ::2] = 0
    c = m - a
    full, _ = oracle.seq_logprob(h, w, tgt, m)
    pa, _ = oracle.seq_logprob(h, w, tgt, a)
    pc, _ = oracle.seq_logprob(h, w, tgt, c)
    assert np.allclose(full, pa + pc, atol=1e-12)
    assert np.all(full < 0)
