"""numpy-facing wrappers around the C oracle (test infrastructure only).

bf16 tensors are ``uint16`` bit patterns.  All results are float64 / int32.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dlm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, OpenMP for the outer loops)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i32, i64, f64, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        lib.oracle_attention_rows.restype = ctypes.c_int
        lib.oracle_attention_rows.argtypes = [vp, i64, i64, i64, vp, vp, i64, i64, i64, vp, vp, vp,
                                              i32, i32, i32, i32, i32, i32, i32, f64, vp, i64, vp, vp]
        lib.oracle_lmhead_rows.restype = ctypes.c_int
        lib.oracle_lmhead_rows.argtypes = [vp, i64, vp, i64, vp, i64, i32, i32, f64, i32, vp,
                                           vp, vp, vp, vp, vp, vp, vp]
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


@dataclass
class KV:
    """One segment of the visible context: k, v are bf16 bits [B, Hkv, len, d];
    pos0 is the absolute position of its first row.  rule (block-causal mode only): "causal" = keys of
    the query's block and earlier ones, "earlier" = earlier blocks only, "same" = the query's block only."""
    k: np.ndarray
    v: np.ndarray
    pos0: int = 0
    rule: str = "causal"

    @property
    def len(self) -> int:
        return self.k.shape[2]


def attention(q: np.ndarray, segments: Sequence[KV], *, mask_mode: str = "full", bs: int = 0,
              q_pos0: int = 0, scale: Optional[float] = None,
              prefix_len_b: Optional[np.ndarray] = None, rows: Optional[np.ndarray] = None):
    """O = softmax(scale * Q K^T) V of a query block against the concatenation of
    the given KV segments (prefix | block | suffix in the rollout).

    q             bf16 bits [B, Lq, Hq, d]
    prefix_len_b  optional [B]: only the first prefix_len_b[b] rows of segments[0] exist
    rows          optional [n, 3] (b, h, i) to evaluate; default all rows
    returns (O, LSE): [n, d], [n] when rows is given, else [B, Lq, Hq, d], [B, Hq, Lq]
    """
    q = np.ascontiguousarray(q, dtype=np.uint16)
    B, Lq, Hq, d = q.shape
    segments = [s for s in segments if s is not None and s.len > 0]
    if segments:
        k = np.ascontiguousarray(np.concatenate([s.k for s in segments], axis=2), dtype=np.uint16)
        v = np.ascontiguousarray(np.concatenate([s.v for s in segments], axis=2), dtype=np.uint16)
        key_pos = np.concatenate([s.pos0 + np.arange(s.len, dtype=np.int32) for s in segments])
        key_rule = np.concatenate([np.full(s.len, {"causal": 0, "earlier": 1, "same": 2}[s.rule], np.int32)
                                   for s in segments])
        Hkv = k.shape[1]
    else:
        Hkv = Hq
        k = np.zeros((B, Hkv, 0, d), dtype=np.uint16)
        v = np.zeros((B, Hkv, 0, d), dtype=np.uint16)
        key_pos = np.zeros((0,), dtype=np.int32)
        key_rule = np.zeros((0,), dtype=np.int32)
    key_pos = np.ascontiguousarray(key_pos, dtype=np.int32)
    key_rule = np.ascontiguousarray(key_rule, dtype=np.int32)
    Lk = k.shape[2]
    key_ok = None
    if prefix_len_b is not None and segments:
        key_ok = np.ones((B, Lk), dtype=np.uint8)
        n0 = segments[0].len
        for b in range(B):
            key_ok[b, int(prefix_len_b[b]):n0] = 0
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    mode = {"full": 0, "block_causal": 1}[mask_mode]
    full = rows is None
    if full:
        bb, ii, hh = np.meshgrid(np.arange(B), np.arange(Lq), np.arange(Hq), indexing="ij")
        rows = np.stack([bb.ravel(), hh.ravel(), ii.ravel()], axis=1)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    n = rows.shape[0]
    out = np.zeros((n, d), dtype=np.float64)
    lse = np.zeros((n,), dtype=np.float64)
    kd = k if Lk else np.zeros((1,), dtype=np.uint16)
    vd = v if Lk else np.zeros((1,), dtype=np.uint16)
    rc = _load().oracle_attention_rows(
        _ptr(q), Lq * Hq * d, Hq * d, d, _ptr(kd), _ptr(vd), Hkv * Lk * d, Lk * d, d,
        _ptr(key_pos), _ptr(key_ok), _ptr(key_rule), Hq, Hkv, d, Lk, mode, int(bs), int(q_pos0), float(scale),
        _ptr(rows), n, _ptr(out), _ptr(lse))
    if rc != 0:
        raise ValueError(f"oracle_attention_rows failed: {rc}")
    if full:
        return out.reshape(B, Lq, Hq, d), lse.reshape(B, Lq, Hq).transpose(0, 2, 1).copy()
    return out, lse


def attention_varlen(q: np.ndarray, k: np.ndarray, v: np.ndarray, cu_seqlens, *, mask_mode: str = "full",
                     bs: int = 0, scale: Optional[float] = None):
    """Packed variable-length attention: the batch is one token-major buffer and sequence b, which owns
    tokens [cu_seqlens[b], cu_seqlens[b+1]), attends only to itself (positions restart at 0 per sequence).

    q bf16 bits [T, Hq, d]; k, v bf16 bits [T, Hkv, d]; returns (O [T, Hq, d], LSE [Hq, T]) in float64.
    """
    T, Hq, d = q.shape
    out = np.zeros((T, Hq, d), np.float64)
    lse = np.zeros((Hq, T), np.float64)
    cu = [int(c) for c in cu_seqlens]
    for b in range(len(cu) - 1):
        a, e = cu[b], cu[b + 1]
        if e <= a:
            continue
        seg = KV(np.ascontiguousarray(k[a:e].transpose(1, 0, 2))[None], np.ascontiguousarray(v[a:e].transpose(1, 0, 2))[None], 0)
        o, l = attention(q[a:e][None], [seg], mask_mode=mask_mode, bs=bs, q_pos0=0, scale=scale)
        out[a:e] = o[0]
        lse[:, a:e] = l[0]
    return out, lse


def lmhead(hidden: np.ndarray, w: np.ndarray, *, row_idx: Optional[np.ndarray] = None,
           inv_temperature: float = 1.0, forbid_token: int = -1,
           target: Optional[np.ndarray] = None):
    """Per row: arg-max token of hidden @ W^T, its softmax probability, LSE, the
    max and the runner-up logit (and the target's logit when targets are given).
    Two alternative confidence scores come with it: `margin` = p(top-1) - p(top-2) and
    `neg_entropy` = sum_v p_v log p_v.

    hidden bf16 bits [R, Dh]; w bf16 bits [V, Dh]; row_idx optional [M] gather.
    returns dict(conf, tok, lse, zmax, z2nd, margin, neg_entropy[, zt]) of length-M arrays.
    """
    hidden = np.ascontiguousarray(hidden, dtype=np.uint16)
    w = np.ascontiguousarray(w, dtype=np.uint16)
    R, Dh = hidden.shape
    V = w.shape[0]
    assert w.shape[1] == Dh
    if row_idx is not None:
        row_idx = np.ascontiguousarray(row_idx, dtype=np.int32)
        M = row_idx.shape[0]
        assert M == 0 or (row_idx.min() >= 0 and row_idx.max() < R)
    else:
        M = R
    conf = np.zeros(M, np.float64)
    tok = np.zeros(M, np.int32)
    lse = np.zeros(M, np.float64)
    zmax = np.zeros(M, np.float64)
    z2nd = np.zeros(M, np.float64)
    nent = np.zeros(M, np.float64)
    zt = None
    if target is not None:
        target = np.ascontiguousarray(target, dtype=np.int32)
        assert target.shape[0] == M and (M == 0 or (target.min() >= 0 and target.max() < V))
        zt = np.zeros(M, np.float64)
    if M:
        rc = _load().oracle_lmhead_rows(_ptr(hidden), Dh, _ptr(row_idx), M, _ptr(w), Dh, Dh, V,
                                        float(inv_temperature), int(forbid_token), _ptr(target),
                                        _ptr(conf), _ptr(tok), _ptr(lse), _ptr(zmax), _ptr(z2nd),
                                        _ptr(zt), _ptr(nent))
        if rc != 0:
            raise ValueError(f"oracle_lmhead_rows failed: {rc}")
    res = dict(conf=conf, tok=tok, lse=lse, zmax=zmax, z2nd=z2nd,
               margin=conf - np.exp(z2nd - lse), neg_entropy=nent)
    if zt is not None:
        res["zt"] = zt
    return res


def block_diffusion_train_attention(q_noisy, k_noisy, v_noisy, q_clean, k_clean, v_clean, *, bs: int,
                                    scale: Optional[float] = None):
    """Attention of one block-diffusion training pass over the pair (noisy x_t, clean x_0) of a sequence
    (Eq. 3: block b of x_t is denoised given itself and the clean blocks before it):
      noisy query in block b  sees noisy keys of block b and clean keys of blocks < b,
      clean query in block b  sees clean keys of blocks <= b.
    q_* bf16 bits [B, L, Hq, d]; k_*, v_* bf16 bits [B, Hkv, L, d].
    returns (O_noisy, LSE_noisy, O_clean, LSE_clean)."""
    On, Ln = attention(q_noisy, [KV(k_clean, v_clean, 0, "earlier"), KV(k_noisy, v_noisy, 0, "same")],
                       mask_mode="block_causal", bs=bs, q_pos0=0, scale=scale)
    Oc, Lc = attention(q_clean, [KV(k_clean, v_clean, 0, "causal")], mask_mode="block_causal", bs=bs, q_pos0=0,
                       scale=scale)
    return On, Ln, Oc, Lc
