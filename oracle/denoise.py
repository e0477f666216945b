"""Selection/commit rule and the block rollout loop of the oracle (test
infrastructure only; plain Python + numpy, no code shared with the HIP path).

The reverse (denoising) process fills a block of masked positions over several
steps; each step evaluates the mask predictor of Eq. (2) on the still-masked
positions and fixes some of them.  Two rules decide which:

  "topk"       the fixed schedule of Section 4.1 (response length / diffusion
               steps tokens per step, e.g. 512/256 = 2): the k most confident
               masked positions commit;
  "threshold"  confidence-threshold parallel decoding (the Fast-dLLM rule the
               paper adopts for rollout): every masked position whose confidence
               is >= tau commits, and the single most confident one always does.

Ties are broken towards the lower index everywhere.
"""
from __future__ import annotations

from typing import Optional, Sequence

import numpy as np

from .ref import KV, attention, lmhead
from .sampling import lmhead_sampled


def select_commit(conf: np.ndarray, mask: np.ndarray, *, rule: str, tau: float = 0.0, k: int = 0,
                  force_top1: bool = True, group_len: Optional[int] = None):
    """Decide which masked positions commit in this step.

    conf   [B, n] confidences (entries at unmasked positions are never looked at)
    mask   [B, n] uint8, 1 = still masked
    Positions are split into consecutive commit groups of group_len (default n: one
    group per sequence); the rule is applied to every group independently.
    returns commit_now uint8 [B, n], n_commit int32 [B], remaining int32 [B]
    """
    conf = np.asarray(conf, dtype=np.float64)
    mask = np.asarray(mask, dtype=np.uint8)
    B, n = mask.shape
    group_len = n if group_len is None else group_len
    assert n % group_len == 0
    commit = np.zeros((B, n), dtype=np.uint8)
    n_commit = np.zeros(B, dtype=np.int32)
    remaining = np.zeros(B, dtype=np.int32)
    for b in range(B):
        for g0 in range(0, n, group_len):
            cand = [i for i in range(g0, g0 + group_len) if mask[b, i]]
            if not cand:
                continue
            if rule == "threshold":
                chosen = [i for i in cand if conf[b, i] >= tau]
                if force_top1:
                    best = cand[0]
                    for i in cand[1:]:
                        if conf[b, i] > conf[b, best]:      # strict: lowest index wins ties
                            best = i
                    if best not in chosen:
                        chosen.append(best)
            elif rule == "topk":
                assert k >= 1
                order = sorted(cand, key=lambda i: (-conf[b, i], i))
                chosen = order[:min(k, len(cand))]
            else:
                raise ValueError(rule)
            for i in chosen:
                commit[b, i] = 1
            n_commit[b] += len(chosen)
            remaining[b] += len(cand) - len(chosen)
    return commit, n_commit, remaining


def apply_commit(x: np.ndarray, x_pos0: int, mask: np.ndarray, tok_dense: np.ndarray,
                 commit: np.ndarray) -> None:
    """x[b, x_pos0 + i] = tok and mask = 0 for committed positions; nothing else changes."""
    B, n = mask.shape
    for b in range(B):
        for i in range(n):
            if commit[b, i]:
                assert mask[b, i] == 1
                x[b, x_pos0 + i] = tok_dense[b, i]
                mask[b, i] = 0


class OracleRollout:
    """Block-by-block rollout of a synthetic workload (see paper_2604_04215_amd.synth).

    Per block: optionally refresh the cache image, then repeat {attention of the
    block against [prefix | block | suffix]; LM head on masked rows; select and
    commit} until nothing is masked.  When a sequence's last masked position
    commits, that step's block K/V is written into its cache slot.
    State (x, mask, cache_k, cache_v) is public so a lock-step checker can re-sync it.
    """

    def __init__(self, cfg, synth, seqs: Optional[Sequence[int]] = None, w: Optional[np.ndarray] = None,
                 sample_seed: Optional[int] = None, sample_stream: int = 0, inv_temperature: float = 1.0,
                 confidence: str = "prob"):
        # confidence: the score the commit rule ranks: "prob" (of the chosen token), "margin" (top-1 minus
        # top-2 probability) or "neg_entropy" (sum p log p); the latter two score the distribution
        self.confidence = confidence
        # sample_seed None: arg-max tokens; else Gumbel-max samples, step s of block b drawing with
        # step counter (b << 16) | s and rows keyed by their index b * Lb + i among ALL B sequences
        self.sample_seed, self.sample_stream, self.inv_temperature = sample_seed, sample_stream, inv_temperature
        self.cfg, self.synth = cfg, synth
        self.seqs = list(range(cfg.B)) if seqs is None else list(seqs)
        self.w = synth.w_vocab(cfg) if w is None else w
        self.x = synth.initial_tokens(cfg, cfg.L, self.seqs)
        self.cache_k, self.cache_v = synth.cache_kv(cfg, 0, self.seqs)
        self.block = -1
        self.step_idx = 0
        self.mask = None

    # geometry of the current block
    @property
    def P(self) -> int:
        return self.cfg.prompt + self.block * self.cfg.Lb

    @property
    def S(self) -> int:
        return self.cfg.L - self.P - self.cfg.Lb if self.cfg.dual_cache else 0

    def snapshot(self) -> dict:
        """Everything needed to resume: a rollout's state is just these buffers and two counters."""
        return dict(x=self.x.copy(), mask=None if self.mask is None else self.mask.copy(),
                    cache_k=self.cache_k.copy(), cache_v=self.cache_v.copy(),
                    block=self.block, step_idx=self.step_idx)

    def restore(self, snap: dict) -> None:
        self.x, self.cache_k, self.cache_v = snap["x"].copy(), snap["cache_k"].copy(), snap["cache_v"].copy()
        self.mask = None if snap["mask"] is None else snap["mask"].copy()
        self.block, self.step_idx = snap["block"], snap["step_idx"]

    def begin_block(self, block: int) -> None:
        cfg = self.cfg
        self.block, self.step_idx = block, 0
        P, Lb = self.P, cfg.Lb
        if cfg.refresh and block > 0:
            k, v = self.synth.cache_kv(cfg, block, self.seqs)
            self.cache_k[:, :, :P] = k[:, :, :P]
            self.cache_v[:, :, :P] = v[:, :, :P]
            if cfg.dual_cache:
                self.cache_k[:, :, P + Lb:] = k[:, :, P + Lb:]
                self.cache_v[:, :, P + Lb:] = v[:, :, P + Lb:]
        self.mask = self.synth.initial_block_mask(cfg, block, self.seqs)

    def segments(self, kb, vb):
        P, Lb, S = self.P, self.cfg.Lb, self.S
        segs = [KV(self.cache_k[:, :, :P], self.cache_v[:, :, :P], 0), KV(kb, vb, P)]
        if S > 0:
            segs.append(KV(self.cache_k[:, :, P + Lb:P + Lb + S], self.cache_v[:, :, P + Lb:P + Lb + S], P + Lb))
        return segs

    def step(self, attn_rows: Optional[np.ndarray] = None) -> dict:
        cfg, syn = self.cfg, self.synth
        n, Lb = len(self.seqs), cfg.Lb
        q = syn.step_q(cfg, self.block, self.step_idx, self.seqs)
        kb, vb = syn.step_kv(cfg, self.block, self.step_idx, self.seqs)
        hid = syn.step_hidden(cfg, self.block, self.step_idx, self.seqs)
        O, lse = attention(q, self.segments(kb, vb), mask_mode=cfg.mask_mode, bs=cfg.bs,
                           q_pos0=self.P, rows=attn_rows)
        mask_before = self.mask.copy()
        row_idx = np.flatnonzero(mask_before.ravel()).astype(np.int32)
        if self.sample_seed is None:
            lm = lmhead(hid.reshape(n * Lb, cfg.Dh), self.w, row_idx=row_idx, forbid_token=cfg.forbid_token,
                        inv_temperature=self.inv_temperature)
        else:
            if self.seqs != list(range(cfg.B)):
                raise ValueError("a sampled rollout keys its noise by row index: run all sequences")
            lm = lmhead_sampled(hid.reshape(n * Lb, cfg.Dh), self.w, row_idx=row_idx,
                                forbid_token=cfg.forbid_token, inv_temperature=self.inv_temperature,
                                seed=self.sample_seed, step=(self.block << 16) | self.step_idx,
                                stream=self.sample_stream)
        if self.confidence != "prob":
            det = lm if self.sample_seed is None else lmhead(hid.reshape(n * Lb, cfg.Dh), self.w, row_idx=row_idx,
                                                             forbid_token=cfg.forbid_token,
                                                             inv_temperature=self.inv_temperature)
            lm = dict(lm, conf=det[self.confidence])
        conf = np.zeros(n * Lb, np.float64)
        tok = np.full(n * Lb, -1, np.int32)
        conf[row_idx] = lm["conf"]
        tok[row_idx] = lm["tok"]
        conf, tok = conf.reshape(n, Lb), tok.reshape(n, Lb)
        commit, n_commit, remaining = select_commit(conf, mask_before, rule=cfg.rule, tau=cfg.tau, k=cfg.k)
        apply_commit(self.x, self.P, self.mask, tok, commit)
        for b in range(n):
            if remaining[b] == 0 and n_commit[b] > 0:     # finished in this very step
                self.cache_k[b, :, self.P:self.P + Lb] = kb[b]
                self.cache_v[b, :, self.P:self.P + Lb] = vb[b]
        out = dict(block=self.block, step=self.step_idx, O=O, lse_attn=lse, row_idx=row_idx, lm=lm,
                   conf=conf, tok=tok, mask_before=mask_before, commit=commit, n_commit=n_commit,
                   remaining=remaining)
        self.step_idx += 1
        return out

    def run(self, blocks: Optional[Sequence[int]] = None, on_step=None) -> dict:
        """Run whole blocks to completion; returns per-block step counts and the commit total."""
        steps, committed = [], 0
        for b in (range(self.cfg.n_blocks) if blocks is None else blocks):
            self.begin_block(b)
            while self.mask.any():
                r = self.step()
                committed += int(r["n_commit"].sum())
                if on_step:
                    on_step(self, r)
            steps.append(self.step_idx)
        return dict(steps=steps, committed=committed)


def full_pass(cfg, synth, seqs: Optional[Sequence[int]] = None, w: Optional[np.ndarray] = None,
              attn_rows: Optional[np.ndarray] = None, lm_rows: Optional[np.ndarray] = None) -> dict:
    """One block-causal full-sequence pass with i.i.d. masking (Eq. 1 / Eq. 3): attention over
    the whole sequence, LM head on masked rows, one threshold commit per block of cfg.bs.

    attn_rows / lm_rows restrict the (expensive) attention and LM-head evaluation to samples;
    with lm_rows given, selection is not evaluated.
    """
    seqs = list(range(cfg.B)) if seqs is None else list(seqs)
    n = len(seqs)
    w = synth.w_vocab(cfg) if w is None else w
    q, k, v = synth.fullpass_qkv(cfg, seqs)
    hid = synth.fullpass_hidden(cfg, seqs)
    mask = synth.fullpass_mask(cfg, seqs)
    O, lse = attention(q, [KV(k, v, 0)], mask_mode="block_causal", bs=cfg.bs, q_pos0=0, rows=attn_rows)
    row_idx = np.flatnonzero(mask.ravel()).astype(np.int32) if lm_rows is None else np.asarray(lm_rows, np.int32)
    lm = lmhead(hid.reshape(n * cfg.L, cfg.Dh), w, row_idx=row_idx, forbid_token=cfg.forbid_token)
    out = dict(O=O, lse_attn=lse, row_idx=row_idx, lm=lm, mask_before=mask.copy())
    if lm_rows is None:
        conf = np.zeros(n * cfg.L, np.float64)
        tok = np.full(n * cfg.L, -1, np.int32)
        conf[row_idx] = lm["conf"]
        tok[row_idx] = lm["tok"]
        conf, tok = conf.reshape(n, cfg.L), tok.reshape(n, cfg.L)
        commit, n_commit, remaining = select_commit(conf, mask, rule="threshold", tau=cfg.tau,
                                                    group_len=cfg.bs)
        x = synth.initial_tokens(cfg, cfg.L, seqs)
        x_before = x.copy()
        apply_commit(x, 0, mask, tok, commit)
        out.update(conf=conf, tok=tok, commit=commit, n_commit=n_commit, remaining=remaining,
                   x_before=x_before, x=x, mask=mask)
    return out


def seq_logprob(hidden, w, target, mask, *, weight=None, forbid_token: int = -1):
    """Masked log-likelihood per sequence: sum over masked positions of log p(target | x_t), the term that the
    NELBO of Eq. (2) / Eq. (3) weights by 1/t.

    hidden bf16 bits [B, n, Dh]; w bf16 bits [V, Dh]; target int [B, n]; mask uint8 [B, n].
    returns (out float64 [B], n_terms int [B]); weight (optional [B]) multiplies each sum.
    """
    B, n, Dh = hidden.shape
    out = np.zeros(B, np.float64)
    n_terms = np.zeros(B, np.int32)
    for b in range(B):
        idx = np.flatnonzero(mask[b]).astype(np.int32)
        n_terms[b] = len(idx)
        if len(idx):
            r = lmhead(hidden[b], w, row_idx=idx, forbid_token=forbid_token, target=np.asarray(target[b])[idx])
            terms = r["zt"] - r["lse"]              # log softmax at the target token
            out[b] = float(np.sum(terms))
        if weight is not None:
            out[b] *= float(weight[b])
    return out, n_terms
