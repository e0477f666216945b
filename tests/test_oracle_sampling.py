"""Pins for the oracle's stochastic token choice (CPU only): the generator against its published
known-answer vectors and a pure-Python big-integer evaluation, the noise against the Gumbel law, and the
sampled tokens against the softmax distribution they must follow (the Gumbel-max identity)."""
import math
import os

import numpy as np
import scipy.stats

import oracle
from oracle import sampling
from paper_2604_04215_amd import synth

HERE = os.path.dirname(os.path.abspath(__file__))


def rnd(seed, shape, std=1.0):
    return synth.normal_bf16(555, 21, (seed,), shape, std)


def f64(u):
    return synth.bf16_bits_to_f64(u)


def test_philox_known_answers():
    n = 0
    for line in open(os.path.join(HERE, "golden", "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        c, k, o = [[int(t, 16) for t in part.split()] for part in line.split("|")]
        got = sampling.philox4x32(np.array(c, dtype=np.uint32), k)
        assert [int(x) for x in got] == o
        n += 1
    assert n == 3


def test_philox_is_a_bijection_with_avalanche():
    # distinct counters give distinct outputs (it is a permutation of the counter space), every output
    # bit is balanced, and flipping one counter bit flips about half of the 128 output bits
    ctr = np.zeros((4096, 4), np.uint32)
    ctr[:, 0] = np.arange(4096)
    out = sampling.philox4x32(ctr, (7, 9))
    assert len({tuple(r) for r in out.tolist()}) == 4096
    bits = np.unpackbits(out.view(np.uint8), axis=1)
    assert np.abs(bits.mean(axis=0) - 0.5).max() < 0.05
    ctr2 = ctr.copy()
    ctr2[:, 1] ^= 1 << 5
    flips = np.unpackbits((out ^ sampling.philox4x32(ctr2, (7, 9))).view(np.uint8), axis=1).sum(axis=1)
    assert abs(flips.mean() - 64) < 1.0
    # the key matters as well
    assert not np.array_equal(out, sampling.philox4x32(ctr, (7, 10)))


def test_uniform_grid_and_gumbel_law():
    assert sampling.uniform_open(np.array([0], np.uint32))[0] == 2.0 ** -24
    assert sampling.uniform_open(np.array([0xFFFFFFFF], np.uint32))[0] == 1.0 - 2.0 ** -24
    assert sampling.uniform_open(np.array([1 << 9], np.uint32))[0] == 3 * 2.0 ** -24
    g = sampling.gumbel_noise(1234, np.arange(8), 50000, step=3, stream=1).ravel()
    assert scipy.stats.kstest(g, "gumbel_r").pvalue > 1e-3
    assert abs(g.mean() - 0.5772156649) < 0.01 and abs(g.var() - math.pi ** 2 / 6) < 0.02


def test_noise_depends_on_every_counter_field_and_on_nothing_else():
    base = sampling.gumbel_noise(99, [5, 6], 103, step=2, stream=4)
    assert base.shape == (2, 103)
    assert np.array_equal(base, sampling.gumbel_noise(99, [5, 6], 103, step=2, stream=4))
    assert np.array_equal(base[1], sampling.gumbel_noise(99, [6], 103, step=2, stream=4)[0])     # keyed by row key only
    assert np.array_equal(base[:, :64], sampling.gumbel_noise(99, [5, 6], 64, step=2, stream=4))  # and by token id
    for other in (sampling.gumbel_noise(98, [5, 6], 103, step=2, stream=4),
                  sampling.gumbel_noise(99, [5, 6], 103, step=3, stream=4),
                  sampling.gumbel_noise(99, [5, 6], 103, step=2, stream=5),
                  sampling.gumbel_noise(99 + (1 << 32), [5, 6], 103, step=2, stream=4)):
        assert not np.any(other == base)
    assert abs(np.corrcoef(base[0], base[1])[0, 1]) < 0.3


def test_sampled_tokens_follow_the_softmax():
    # one hidden row, many independent draws (one per step): token frequencies must match softmax(z / T)
    Dh, V, n = 32, 12, 20000
    h, w = rnd(1, (1, Dh)), rnd(2, (V, Dh), 0.35)
    inv_t = 0.8
    z = (f64(h) @ f64(w).T)[0] * inv_t
    z[3] = -np.inf
    p = np.exp(z - z.max())
    p /= p.sum()
    counts = np.zeros(V)
    confs = []
    for step in range(n // 50):
        hh = np.repeat(h, 50, axis=0)                     # 50 copies of the row: 50 row keys, 50 independent draws
        r = sampling.lmhead_sampled(hh, w, seed=2024, step=step, inv_temperature=inv_t, forbid_token=3)
        counts += np.bincount(r["tok"], minlength=V)
        confs.append((r["tok"], r["conf"]))
    assert counts[3] == 0
    keep = p > 0
    assert scipy.stats.chisquare(counts[keep], p[keep] * n).pvalue > 1e-3
    tok, conf = confs[0]
    assert np.allclose(conf, p[tok], atol=1e-12)          # confidence = probability of the token that was drawn


def test_sampling_agrees_with_the_deterministic_head_on_shared_outputs():
    M, Dh, V = 9, 64, 301
    h, w = rnd(3, (20, Dh)), rnd(4, (V, Dh), 0.4)
    idx = np.array([0, 19, 7, 3, 4, 11, 12, 13, 2], np.int32)
    r = sampling.lmhead_sampled(h, w, seed=5, step=1, stream=2, row_idx=idx, forbid_token=V - 1)
    d = oracle.lmhead(h, w, row_idx=idx, forbid_token=V - 1, target=r["tok"])
    assert np.allclose(r["lse"], d["lse"], atol=1e-11) and np.allclose(r["zmax"], d["zmax"], atol=1e-11)
    assert np.allclose(r["ztok"], d["zt"], atol=1e-11)
    assert np.allclose(np.log(r["conf"]), d["zt"] - d["lse"], atol=1e-11)
    assert np.all(r["pmax"] >= r["p2nd"]) and np.all(r["tok"] != V - 1)
    # noise is keyed by the row's index in `hidden`: gathering in another order permutes the result
    perm = np.array([4, 0, 8, 2, 1, 3, 7, 6, 5])
    r2 = sampling.lmhead_sampled(h, w, seed=5, step=1, stream=2, row_idx=idx[perm], forbid_token=V - 1)
    assert np.array_equal(r2["tok"], r["tok"][perm])
    # a very low temperature (large inverse) makes sampling greedy
    cold = sampling.lmhead_sampled(h, w, seed=5, row_idx=idx, inv_temperature=200.0)
    greedy = oracle.lmhead(h, w, row_idx=idx, inv_temperature=200.0)
    assert np.array_equal(cold["tok"], greedy["tok"])
