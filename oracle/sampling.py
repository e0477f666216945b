"""Stochastic token choice for the rollout (TEST INFRASTRUCTURE ONLY, like the rest of this package).

Sampling a token from softmax(z) is done with the Gumbel-max identity: with independent standard
Gumbel noise g_v, arg max_v (z_v + g_v) is distributed as softmax(z).  The noise has to be the same
on both sides of a parity test, so it comes from a counter-based generator that each side implements
for itself: Philox-4x32 with ten rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
as 1, 2, 3", SC 2011), keyed by the 64-bit seed and counted by (vocabulary quad, row key, step, stream).

Stochastic rollouts are what the RL recipes need (Section 4.1, implementation details: a group of 8
rollouts per prompt); the paper does not say how the noise is generated.
"""
from __future__ import annotations

from typing import Optional

import numpy as np

_M0, _M1 = 0xD2511F53, 0xCD9E8D57          # round multipliers
_W0, _W1 = 0x9E3779B9, 0xBB67AE85          # key increments (golden ratio, sqrt(3) - 1)
_MASK32 = np.uint64(0xFFFFFFFF)


def philox4x32(counter: np.ndarray, key, rounds: int = 10) -> np.ndarray:
    """counter uint32 [..., 4], key (k0, k1) -> uint32 [..., 4]."""
    c = [np.asarray(counter[..., i], dtype=np.uint64) for i in range(4)]
    k0, k1 = int(key[0]) & 0xFFFFFFFF, int(key[1]) & 0xFFFFFFFF
    for _ in range(rounds):
        p0 = np.uint64(_M0) * c[0]          # 32 x 32 -> 64 bit products
        p1 = np.uint64(_M1) * c[2]
        hi0, lo0 = p0 >> np.uint64(32), p0 & _MASK32
        hi1, lo1 = p1 >> np.uint64(32), p1 & _MASK32
        c = [hi1 ^ c[1] ^ np.uint64(k0), lo1, hi0 ^ c[3] ^ np.uint64(k1), lo0]
        k0, k1 = (k0 + _W0) & 0xFFFFFFFF, (k1 + _W1) & 0xFFFFFFFF
    return np.stack(c, axis=-1).astype(np.uint32)


def uniform_open(bits: np.ndarray) -> np.ndarray:
    """The top 23 bits k of a word give u = (2k + 1) / 2^24 in (0, 1): an odd 24-bit numerator, so u
    and 1 - u are exact in single precision as well."""
    k = np.asarray(bits, dtype=np.uint64) >> np.uint64(9)
    return (2.0 * k.astype(np.float64) + 1.0) / 16777216.0


def gumbel_noise(seed: int, row_keys, V: int, step: int = 0, stream: int = 0) -> np.ndarray:
    """Standard Gumbel noise float64 [len(row_keys), V]: the word for (row key r, token v) is word v % 4 of
    Philox(counter = (v // 4, r, step, stream), key = (seed low 32 bits, seed high 32 bits))."""
    row_keys = np.asarray(row_keys, dtype=np.uint32)
    nq = (V + 3) // 4
    ctr = np.zeros((len(row_keys), nq, 4), dtype=np.uint32)
    ctr[..., 0] = np.arange(nq, dtype=np.uint32)[None, :]
    ctr[..., 1] = row_keys[:, None]
    ctr[..., 2] = np.uint32(step & 0xFFFFFFFF)
    ctr[..., 3] = np.uint32(stream & 0xFFFFFFFF)
    words = philox4x32(ctr, (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)).reshape(len(row_keys), nq * 4)[:, :V]
    return -np.log(-np.log(uniform_open(words)))


def _bf16_to_f64(u16: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(u16, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def lmhead_sampled(hidden: np.ndarray, w: np.ndarray, *, seed: int, step: int = 0, stream: int = 0,
                   row_idx: Optional[np.ndarray] = None, inv_temperature: float = 1.0, forbid_token: int = -1):
    """Per selected row: z = (hidden . W^T) * inv_temperature (forbidden token at -inf), token =
    arg max_v (z_v + g_v) with the noise keyed by the row's index in `hidden`, confidence = softmax(z) at
    that token.  Also returns the log-sum-exp, the perturbed maximum and its runner-up (the margin that says
    whether single-precision arithmetic could have picked another token).

    hidden bf16 bits [R, Dh]; w bf16 bits [V, Dh]; row_idx optional [M].  Logits are materialised
    ([M, V] float64): meant for small M.
    """
    R = hidden.shape[0]
    rows = np.arange(R, dtype=np.int64) if row_idx is None else np.asarray(row_idx, dtype=np.int64)
    V = w.shape[0]
    hf = _bf16_to_f64(hidden)[rows]
    z = np.empty((len(rows), V), np.float64)
    for v0 in range(0, V, 8192):                          # vocabulary slabs only bound the float64 copy of W
        z[:, v0:v0 + 8192] = hf @ _bf16_to_f64(w[v0:v0 + 8192]).T
    z *= float(inv_temperature)
    if forbid_token >= 0:
        z[:, forbid_token] = -np.inf
    zmax = z.max(axis=1)
    lse = zmax + np.log(np.exp(z - zmax[:, None]).sum(axis=1))
    pert = z + gumbel_noise(seed, rows, V, step, stream)
    tok = pert.argmax(axis=1).astype(np.int32)            # first index on (measure-zero) ties
    m = len(rows)
    ztok = z[np.arange(m), tok]
    top2 = np.partition(pert, V - 2, axis=1)[:, V - 2:] if V >= 2 else np.stack([np.full(m, -np.inf), pert[:, 0]], 1)
    return dict(tok=tok, conf=np.exp(ztok - lse), lse=lse, zmax=zmax, ztok=ztok, pmax=top2[:, 1], p2nd=top2[:, 0])
