"""Gradient of block attention (TEST INFRASTRUCTURE ONLY, like the rest of this package).

For O = softmax(scale * Q K^T + mask) V and an upstream gradient dO, with P the softmax matrix:
    dV = P^T dO,    dP = dO V^T,    dS = P * (dP - rowsum(dP * P)),    dQ = scale * dS K,    dK = scale * dS^T Q
(the derivative of a row-wise softmax is diag(p) - p p^T).  With grouped-query heads the gradients of a KV
head sum over the query heads that share it.  This is what training a mask predictor through Eq. 2 / Eq. 3
needs from the attention layers; the visibility rules are the ones of the forward pass.
Everything is dense float64 numpy: meant for sizes the tests use.
"""
from __future__ import annotations

import math
from typing import Optional, Sequence

import numpy as np

from .ref import KV

_RULE = {"causal": 0, "earlier": 1, "same": 2}


def _f64(u16: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(u16, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def visibility(Lq: int, segments: Sequence[KV], *, mask_mode: str, bs: int, q_pos0: int) -> np.ndarray:
    """bool [Lq, Lk]: may query row i see key j of the concatenated segments."""
    key_pos = np.concatenate([s.pos0 + np.arange(s.len) for s in segments]) if segments else np.zeros(0, int)
    if mask_mode == "full":
        return np.ones((Lq, len(key_pos)), bool)
    rule = np.concatenate([np.full(s.len, _RULE[s.rule]) for s in segments])
    kb = (key_pos // bs)[None, :]
    qb = ((q_pos0 + np.arange(Lq)) // bs)[:, None]
    return np.where(rule[None, :] == 0, kb <= qb, np.where(rule[None, :] == 1, kb < qb, kb == qb))


def attention_backward(q: np.ndarray, segments: Sequence[KV], d_out: np.ndarray, *, mask_mode: str = "full",
                       bs: int = 0, q_pos0: int = 0, scale: Optional[float] = None):
    """q, d_out bf16 bits [B, Lq, Hq, d]; segments as in the forward oracle.
    returns (dQ [B, Lq, Hq, d], [(dK_s, dV_s) per segment, each [B, Hkv, len_s, d]]) in float64."""
    segments = [s for s in segments if s is not None and s.len > 0]
    B, Lq, Hq, d = q.shape
    Q, dO = _f64(q), _f64(d_out)
    K = np.concatenate([_f64(s.k) for s in segments], axis=2)
    V = np.concatenate([_f64(s.v) for s in segments], axis=2)
    Hkv, Lk = K.shape[1], K.shape[2]
    g = Hq // Hkv
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    vis = visibility(Lq, segments, mask_mode=mask_mode, bs=bs, q_pos0=q_pos0)
    dQ = np.zeros((B, Lq, Hq, d))
    dK = np.zeros((B, Hkv, Lk, d))
    dV = np.zeros((B, Hkv, Lk, d))
    for b in range(B):
        for h in range(Hq):
            kh = h // g
            s = np.where(vis, scale * (Q[b, :, h] @ K[b, kh].T), -np.inf)
            m = s.max(axis=1, keepdims=True)
            m = np.where(np.isfinite(m), m, 0.0)                    # a row that sees no key: P = 0, no gradient
            e = np.exp(s - m)
            den = e.sum(axis=1, keepdims=True)
            P = np.divide(e, den, out=np.zeros_like(e), where=den > 0)
            dV[b, kh] += P.T @ dO[b, :, h]
            dP = dO[b, :, h] @ V[b, kh].T
            dS = P * (dP - (dP * P).sum(axis=1, keepdims=True))
            dQ[b, :, h] = scale * (dS @ K[b, kh])
            dK[b, kh] += scale * (dS.T @ Q[b, :, h])
    out, a = [], 0
    for sg in segments:
        out.append((dK[:, :, a:a + sg.len], dV[:, :, a:a + sg.len]))
        a += sg.len
    return dQ, out
