"""Seeded synthetic inputs for the dLLM rollout denoising step.

This module only *draws* inputs: shapes, seeds, normal draws rounded to bf16 bit
patterns, and random masking patterns.  It contains none of the arithmetic of
the denoising step (no attention, no softmax, no selection) and is the one
module that both the HIP path's callers and the CPU oracle's callers may use,
so that both see bit-identical inputs.

Every tensor is a pure function of ``(seed, tensor tag, index tuple, sequence
index)`` through a counter-based Philox stream, so a sequence's data does not
depend on the batch size or on the order in which tensors are requested.

The shapes follow the rollout settings of the paper's Section 4.1 (block length
32, rollout group 8, responses of 256/512 tokens) on LLaDA-8B-, Dream-7B- and
SDAR/LLaDA2-like head geometries; the i.i.d. masking of the full-sequence pass
follows the forward process of Eq. (1) with alpha_t = 0.5.  bf16 values are kept
as ``uint16`` bit patterns on the host.
"""
from __future__ import annotations

import dataclasses
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Dict, Tuple

import numpy as np

MASK64 = (1 << 64) - 1

# tensor tags
TAG_Q, TAG_KBLK, TAG_VBLK, TAG_HIDDEN, TAG_W, TAG_KCACHE, TAG_VCACHE, TAG_MASK, TAG_X = range(1, 10)

W_CHUNK_ROWS = 1024  # W_vocab is drawn in fixed chunks of rows so any caller gets the same bits
_WORKERS = max(1, min(16, os.cpu_count() or 1))   # independent streams are drawn in parallel threads


def _pmap(fn, items):
    items = list(items)
    if len(items) <= 1 or _WORKERS == 1:
        return [fn(i) for i in items]
    with ThreadPoolExecutor(max_workers=_WORKERS) as ex:
        return list(ex.map(fn, items))


# --------------------------------------------------------------------------- #
# bf16 <-> float helpers (format conversion only)
# --------------------------------------------------------------------------- #
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even), return uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    nan = np.isnan(x)
    rounding = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = ((u + rounding) >> np.uint32(16)).astype(np.uint16)
    if nan.any():
        r = np.where(nan, np.uint16(0x7FC0), r)
    return r


def bf16_bits_to_f32(u16: np.ndarray) -> np.ndarray:
    u16 = np.ascontiguousarray(u16, dtype=np.uint16)
    return (u16.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(u16: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(u16).astype(np.float64)


# --------------------------------------------------------------------------- #
# counter-based streams
# --------------------------------------------------------------------------- #
def _mix(*ints: int) -> int:
    """64-bit hash of a tuple of small integers (splitmix64 finaliser, chained)."""
    h = 0x9E3779B97F4A7C15
    for v in ints:
        h = (h ^ (int(v) & MASK64)) & MASK64
        h = (h + 0x9E3779B97F4A7C15) & MASK64
        z = h
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
        h = z ^ (z >> 31)
    return h


def stream(seed: int, tag: int, *idx: int) -> np.random.Generator:
    key = np.array([int(seed) & MASK64, _mix(tag, *idx)], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def normal_bf16(seed: int, tag: int, idx: Tuple[int, ...], shape, std: float = 1.0) -> np.ndarray:
    g = stream(seed, tag, *idx)
    x = g.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return f32_to_bf16_bits(x)


# --------------------------------------------------------------------------- #
# workload description
# --------------------------------------------------------------------------- #
@dataclass(frozen=True)
class Config:
    """One synthetic rollout workload.

    prompt/gen/Lb   prompt length, generated length, denoising block length
    rule            "threshold" (commit conf >= tau, plus the most confident one)
                    or "topk" (commit the k most confident per step)
    dual_cache      the query block also attends to a cached suffix (future blocks)
    mask_mode       "full" (bidirectional) or "block_causal" with block size bs
    refresh         prefix (and suffix) cache is overwritten with fresh K/V at
                    the start of every block
    w_dist          "var": W ~ N(0, variance Dh^-1/2); "std": W ~ N(0, std Dh^-1/2)
    init_masked     number of masked positions in the first block (None = all)
    """
    name: str
    B: int
    Hq: int
    Hkv: int
    d: int
    Dh: int
    V: int
    prompt: int
    gen: int
    Lb: int
    rule: str = "threshold"
    tau: float = 0.9
    k: int = 0
    dual_cache: bool = False
    mask_mode: str = "full"
    bs: int = 0
    refresh: bool = True
    w_dist: str = "var"
    init_masked: int | None = None
    seed: int = 20260415

    @property
    def n_blocks(self) -> int:
        return self.gen // self.Lb

    @property
    def L(self) -> int:
        return self.prompt + self.gen

    @property
    def forbid_token(self) -> int:
        return self.V - 1  # stands in for the <MASK> id: never predicted

    @property
    def w_std(self) -> float:
        return self.Dh ** -0.25 if self.w_dist == "var" else self.Dh ** -0.5

    def replace(self, **kw) -> "Config":
        return dataclasses.replace(self, **kw)


CONFIGS: Dict[str, Config] = {
    # the five benchmark workloads
    "c1": Config("c1", B=1, Hq=4, Hkv=4, d=64, Dh=256, V=2048, prompt=256, gen=32, Lb=32,
                 rule="threshold", tau=0.9, init_masked=16, refresh=False, seed=20260415 + 1),
    "c2": Config("c2", B=8, Hq=32, Hkv=32, d=128, Dh=4096, V=126464, prompt=512, gen=256, Lb=32,
                 rule="threshold", tau=0.9, refresh=True, seed=20260415 + 2),
    "c3": Config("c3", B=16, Hq=32, Hkv=32, d=128, Dh=4096, V=126464, prompt=1024, gen=512, Lb=32,
                 rule="threshold", tau=0.9, dual_cache=True, refresh=True, seed=20260415 + 3),
    "c4": Config("c4", B=32, Hq=28, Hkv=4, d=128, Dh=3584, V=152064, prompt=768, gen=256, Lb=32,
                 rule="topk", k=4, refresh=False, seed=20260415 + 4),
    "c5a": Config("c5a", B=64, Hq=32, Hkv=8, d=128, Dh=4096, V=157184, prompt=4092, gen=4, Lb=4,
                  rule="threshold", tau=0.95, mask_mode="block_causal", bs=4, refresh=False,
                  seed=20260415 + 5),
    # scaled-down twins (same structure, sizes a CPU finishes in seconds; ragged on purpose)
    "mini2": Config("mini2", B=2, Hq=4, Hkv=4, d=128, Dh=256, V=1000, prompt=72, gen=64, Lb=32,
                    rule="threshold", tau=0.9, refresh=True, seed=777 + 2),
    "mini3": Config("mini3", B=3, Hq=4, Hkv=4, d=128, Dh=192, V=777, prompt=100, gen=96, Lb=32,
                    rule="threshold", tau=0.9, dual_cache=True, refresh=True, seed=777 + 3),
    "mini4": Config("mini4", B=2, Hq=14, Hkv=2, d=128, Dh=320, V=1500, prompt=40, gen=64, Lb=32,
                    rule="topk", k=4, refresh=False, seed=777 + 4),
    "mini5a": Config("mini5a", B=3, Hq=8, Hkv=2, d=128, Dh=256, V=900, prompt=188, gen=12, Lb=4,
                     rule="threshold", tau=0.95, mask_mode="block_causal", bs=4, refresh=False,
                     seed=777 + 5),
    "mini1": Config("mini1", B=1, Hq=2, Hkv=2, d=64, Dh=64, V=300, prompt=40, gen=32, Lb=32,
                    rule="threshold", tau=0.9, init_masked=16, refresh=False, seed=777 + 1),
}


@dataclass(frozen=True)
class FullPassConfig:
    """Full-sequence block-causal pass with Bernoulli masking (training-style)."""
    name: str
    B: int
    Hq: int
    Hkv: int
    d: int
    Dh: int
    V: int
    L: int
    bs: int
    tau: float = 0.95
    mask_prob: float = 0.5
    w_dist: str = "var"
    seed: int = 20260415 + 6

    @property
    def forbid_token(self) -> int:
        return self.V - 1

    @property
    def w_std(self) -> float:
        return self.Dh ** -0.25 if self.w_dist == "var" else self.Dh ** -0.5

    def replace(self, **kw) -> "FullPassConfig":
        return dataclasses.replace(self, **kw)


FULLPASS: Dict[str, FullPassConfig] = {
    "c5b": FullPassConfig("c5b", B=64, Hq=32, Hkv=8, d=128, Dh=4096, V=157184, L=4096, bs=4),
    "mini5b": FullPassConfig("mini5b", B=2, Hq=4, Hkv=2, d=128, Dh=128, V=500, L=204, bs=4,
                             seed=777 + 6),
}


# --------------------------------------------------------------------------- #
# tensors
# --------------------------------------------------------------------------- #
def w_vocab(cfg, rows: slice | None = None) -> np.ndarray:
    """W_vocab [V, Dh] bf16 bits (or the requested row range)."""
    lo, hi = (0, cfg.V) if rows is None else (rows.start or 0, cfg.V if rows.stop is None else rows.stop)
    out = np.empty((hi - lo, cfg.Dh), dtype=np.uint16)
    c0, c1 = lo // W_CHUNK_ROWS, (hi + W_CHUNK_ROWS - 1) // W_CHUNK_ROWS

    def one(c):
        r0, r1 = c * W_CHUNK_ROWS, min((c + 1) * W_CHUNK_ROWS, cfg.V)
        blk = normal_bf16(cfg.seed, TAG_W, (c,), (r1 - r0, cfg.Dh), cfg.w_std)
        a, b = max(r0, lo), min(r1, hi)
        out[a - lo:b - lo] = blk[a - r0:b - r0]

    _pmap(one, range(c0, c1))
    return out


def _per_seq(cfg, tag: int, idx: Tuple[int, ...], shape_one, std: float = 1.0, seqs=None) -> np.ndarray:
    seqs = list(range(cfg.B) if seqs is None else seqs)
    out = np.empty((len(seqs),) + tuple(shape_one), dtype=np.uint16)

    def one(n):
        out[n] = normal_bf16(cfg.seed, tag, idx + (seqs[n],), shape_one, std)

    _pmap(one, range(len(seqs)))
    return out


def step_q(cfg: Config, block: int, step: int, seqs=None) -> np.ndarray:
    """Q for the block's positions: [B, Lb, Hq, d]."""
    return _per_seq(cfg, TAG_Q, (block, step), (cfg.Lb, cfg.Hq, cfg.d), seqs=seqs)


def step_kv(cfg: Config, block: int, step: int, seqs=None):
    """The block's own K and V: each [B, Hkv, Lb, d]."""
    k = _per_seq(cfg, TAG_KBLK, (block, step), (cfg.Hkv, cfg.Lb, cfg.d), seqs=seqs)
    v = _per_seq(cfg, TAG_VBLK, (block, step), (cfg.Hkv, cfg.Lb, cfg.d), seqs=seqs)
    return k, v


def step_hidden(cfg: Config, block: int, step: int, seqs=None) -> np.ndarray:
    """Final hidden state of the block's positions: [B, Lb, Dh]."""
    return _per_seq(cfg, TAG_HIDDEN, (block, step), (cfg.Lb, cfg.Dh), seqs=seqs)


def cache_kv(cfg: Config, version: int, seqs=None):
    """A full-sequence K/V cache image [B, Hkv, L, d] (what a refresh at block
    `version` installs; version 0 is the initial prompt cache)."""
    k = _per_seq(cfg, TAG_KCACHE, (version,), (cfg.Hkv, cfg.L, cfg.d), seqs=seqs)
    v = _per_seq(cfg, TAG_VCACHE, (version,), (cfg.Hkv, cfg.L, cfg.d), seqs=seqs)
    return k, v


def initial_block_mask(cfg: Config, block: int, seqs=None) -> np.ndarray:
    """uint8 [B, Lb]; 1 = masked.  All masked unless cfg.init_masked says otherwise
    (then the first init_masked entries of a seeded permutation of the block)."""
    seqs = range(cfg.B) if seqs is None else seqs
    out = np.ones((len(seqs), cfg.Lb), dtype=np.uint8)
    if cfg.init_masked is not None and cfg.init_masked < cfg.Lb:
        for n, b in enumerate(seqs):
            perm = stream(cfg.seed, TAG_MASK, block, b).permutation(cfg.Lb)
            out[n] = 0
            out[n, perm[:cfg.init_masked]] = 1
    return out


def initial_tokens(cfg, L: int, seqs=None) -> np.ndarray:
    """int32 [B, L] token buffer before any commit (arbitrary known ids < V-1)."""
    seqs = range(cfg.B) if seqs is None else seqs
    return np.stack([stream(cfg.seed, TAG_X, b).integers(0, cfg.V - 1, size=L, dtype=np.int32)
                     for b in seqs])


# full-sequence pass -------------------------------------------------------- #
def fullpass_qkv(cfg: FullPassConfig, seqs=None):
    """Q [B, L, Hq, d], K, V [B, Hkv, L, d]."""
    q = _per_seq(cfg, TAG_Q, (0, 0), (cfg.L, cfg.Hq, cfg.d), seqs=seqs)
    k = _per_seq(cfg, TAG_KBLK, (0, 0), (cfg.Hkv, cfg.L, cfg.d), seqs=seqs)
    v = _per_seq(cfg, TAG_VBLK, (0, 0), (cfg.Hkv, cfg.L, cfg.d), seqs=seqs)
    return q, k, v


def fullpass_hidden(cfg: FullPassConfig, seqs=None) -> np.ndarray:
    """[B, L, Dh]."""
    return _per_seq(cfg, TAG_HIDDEN, (0, 0), (cfg.L, cfg.Dh), seqs=seqs)


def fullpass_mask(cfg: FullPassConfig, seqs=None) -> np.ndarray:
    """uint8 [B, L]: each position masked independently with probability mask_prob."""
    seqs = range(cfg.B) if seqs is None else seqs
    return np.stack([(stream(cfg.seed, TAG_MASK, 0, b).random(cfg.L) < cfg.mask_prob).astype(np.uint8)
                     for b in seqs])


# packed variable-length batch ---------------------------------------------- #
@dataclass(frozen=True)
class VarlenConfig:
    """Packed batch for padding-free bidirectional attention: B sequences, each a prompt of
    prompt_lo..prompt_hi tokens followed by a response cut at its end-of-sequence token
    (resp_lo..resp_hi valid tokens), laid out back to back without PAD rows."""
    name: str
    B: int
    Hq: int
    Hkv: int
    d: int
    prompt_lo: int
    prompt_hi: int
    resp_lo: int
    resp_hi: int
    seed: int = 20260415 + 7

    @property
    def max_len(self) -> int:
        return self.prompt_hi + self.resp_hi

    def replace(self, **kw) -> "VarlenConfig":
        return dataclasses.replace(self, **kw)


TAG_LEN = 10

VARLEN: Dict[str, VarlenConfig] = {
    # 8B-class masked diffusion LM heads (32 x 128), GSM8K-like prompts + responses up to 512 tokens
    "v1": VarlenConfig("v1", B=128, Hq=32, Hkv=32, d=128, prompt_lo=64, prompt_hi=384, resp_lo=32, resp_hi=512),
    # grouped-query variant (7B-class, 28 query / 4 KV heads)
    "v2": VarlenConfig("v2", B=128, Hq=28, Hkv=4, d=128, prompt_lo=64, prompt_hi=384, resp_lo=32, resp_hi=512),
    "miniv1": VarlenConfig("miniv1", B=7, Hq=4, Hkv=2, d=64, prompt_lo=1, prompt_hi=40, resp_lo=0, resp_hi=130,
                           seed=777 + 7),
}


def varlen_seqlens(cfg: VarlenConfig) -> np.ndarray:
    """int32 [B]: prompt + valid response length of every sequence (uniform in the configured ranges)."""
    g = stream(cfg.seed, TAG_LEN, 0)
    prompt = g.integers(cfg.prompt_lo, cfg.prompt_hi + 1, cfg.B)
    resp = g.integers(cfg.resp_lo, cfg.resp_hi + 1, cfg.B)
    return (prompt + resp).astype(np.int32)


def varlen_cu_seqlens(cfg: VarlenConfig) -> np.ndarray:
    """int32 [B + 1]: exclusive prefix sum of varlen_seqlens (token offset of each sequence)."""
    return np.concatenate([[0], np.cumsum(varlen_seqlens(cfg))]).astype(np.int32)


def varlen_qkv(cfg: VarlenConfig):
    """Q [T, Hq, d], K, V [T, Hkv, d] for the packed batch (T = total tokens)."""
    cu = varlen_cu_seqlens(cfg)
    T = int(cu[-1])
    q = np.empty((T, cfg.Hq, cfg.d), np.uint16)
    k = np.empty((T, cfg.Hkv, cfg.d), np.uint16)
    v = np.empty((T, cfg.Hkv, cfg.d), np.uint16)

    def one(b):
        a, e = int(cu[b]), int(cu[b + 1])
        q[a:e] = normal_bf16(cfg.seed, TAG_Q, (1, b), (e - a, cfg.Hq, cfg.d))
        k[a:e] = normal_bf16(cfg.seed, TAG_KBLK, (1, b), (e - a, cfg.Hkv, cfg.d))
        v[a:e] = normal_bf16(cfg.seed, TAG_VBLK, (1, b), (e - a, cfg.Hkv, cfg.d))

    _pmap(one, range(cfg.B))
    return q, k, v, cu
