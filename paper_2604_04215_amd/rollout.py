"""Block rollout driver on top of the libdlm binding.

Owns the device-side state of a rollout (token buffer, block mask, KV cache,
per-step outputs) and enqueues the three calls of one denoising step.  All
arithmetic happens inside libdlm's kernels; this module only wires buffers.

Loop control: the commit kernel leaves the compacted list of still-masked rows
and its length on the device, and the next LM-head call reads that length from
the device, so a step never needs a host round trip to size its work.  The
host only has to learn when a block is finished; `run_block` polls `remaining`
one step late (the result of step s-1 is read after step s has been queued), so
the GPU never idles waiting for the host.  With the total the commit kernel
also reports the largest per-sequence count: when that is no more than the next
step is certain to commit, the step already queued is the block's last, and
the loop neither queues an empty step behind it nor waits for it.
"""
from __future__ import annotations

import ctypes as C
import time
from typing import Callable, Optional

import torch

from . import binding as dlm

_RULES = {"threshold": dlm.RULE_THRESHOLD, "topk": dlm.RULE_TOPK}
_MASKS = {"full": dlm.MASK_FULL, "block_causal": dlm.MASK_BLOCK_CAUSAL}


class StepPoll:
    """Where the host learns what one queued step left masked: one int32 of pinned host memory that the step's commit
    kernel overwrites, with a system-scope store, with the number of positions still masked.  The host sets the word
    to -1 before it queues the step and watches until the device's value (>= 0) shows.  Nothing sits in the queue
    between one step's kernels and the next step's: an event recorded after every step put 5 - 6 us between the
    commit kernel and the next attention kernel on MI355X (kernel trace), this costs the queue nothing."""

    TIMEOUT_S = 60.0

    def __init__(self):
        # [0]: positions still masked in all sequences together; [1]: the most any one sequence still has (stored by the
        # kernel before [0], so it is there once [0] is)
        self.words = torch.zeros(2, dtype=torch.int32).pin_memory()
        self.word, self.word_max = self.words[0:1], self.words[1:2]
        self.view = self.words.numpy()         # shares the pinned memory; every read is a load from it
        self.ptr, self.ptr_max = self.word.data_ptr(), self.word_max.data_ptr()

    def arm(self) -> None:
        self.view[0] = -1

    @property
    def left_max(self) -> int:
        """After wait(): the largest per-sequence count of still-masked positions that the step left."""
        return int(self.view[1])

    def wait(self) -> int:
        """Blocks (spinning) until the step's commit kernel has stored its count; raises if none shows in TIMEOUT_S."""
        view = self.view
        t0 = None
        while True:
            for _ in range(4096):
                v = int(view[0])
                if v >= 0:
                    return v
            now = time.perf_counter()
            if t0 is None:
                t0 = now
            elif now - t0 > self.TIMEOUT_S:
                raise RuntimeError(f"no result of a queued denoising step within {self.TIMEOUT_S:.0f} s "
                                   "(did its dlm_unmask_commit launch fail?)")


class GpuRollout:
    def __init__(self, cfg, w: torch.Tensor, device: str = "cuda:0", record_steps: bool = False,
                 sample_seed: Optional[int] = None, sample_stream: int = 0, inv_temperature: float = 1.0,
                 confidence: str = "prob"):
        """sample_seed None: greedy (arg-max) tokens.  An integer: tokens are sampled from the softmax at
        inv_temperature; step s of block b draws with sample_step = (b << 16) | s, so no two steps of a
        rollout share noise, and rollouts of one prompt differ by sample_stream."""
        self.cfg, self.dev = cfg, torch.device(device)
        self._dev_index = self.dev.index if self.dev.index is not None else torch.cuda.current_device()
        self.sample_seed, self.sample_stream, self.inv_temperature = sample_seed, sample_stream, inv_temperature
        # which score the commit rule ranks: token probability, top-2 margin or negative entropy
        self.conf_mode = {"prob": dlm.CONF_TOKEN_PROB, "margin": dlm.CONF_MARGIN, "neg_entropy": dlm.CONF_NEG_ENTROPY}[confidence]
        B, Lb, L = cfg.B, cfg.Lb, cfg.L
        dev = self.dev
        self.w = w
        self.x = torch.zeros((B, L), dtype=torch.int32, device=dev)
        self.mask = torch.zeros((B, Lb), dtype=torch.uint8, device=dev)
        self.cache_k = torch.zeros((B, cfg.Hkv, L, cfg.d), dtype=torch.bfloat16, device=dev)
        self.cache_v = torch.zeros_like(self.cache_k)
        self.O = torch.zeros((B, Lb, cfg.Hq, cfg.d), dtype=torch.bfloat16, device=dev)
        self.lse_attn = torch.zeros((B, cfg.Hq, Lb), dtype=torch.float32, device=dev)
        n = B * Lb
        self.conf = torch.zeros((B, Lb), dtype=torch.float32, device=dev)
        self.tok = torch.zeros((B, Lb), dtype=torch.int32, device=dev)
        self.lse = torch.zeros(n, dtype=torch.float32, device=dev)
        self.zmax = torch.zeros(n, dtype=torch.float32, device=dev)
        self.z2nd = torch.zeros(n, dtype=torch.float32, device=dev)
        self.commit_now = torch.zeros((B, Lb), dtype=torch.uint8, device=dev)
        self.n_commit = torch.zeros(B, dtype=torch.int32, device=dev)
        # two buffers: a step's write-back reads the previous step's counts while its selection writes the new ones
        self._remaining2 = [torch.zeros(B, dtype=torch.int32, device=dev) for _ in range(2)]
        self.remaining = self._remaining2[0]     # the counts written by the step queued last
        self.row_idx = torch.zeros(n, dtype=torch.int32, device=dev)
        self.m_dev = torch.zeros(1, dtype=torch.int32, device=dev)
        self.commit_step = torch.full((B, Lb), -1, dtype=torch.int16, device=dev) if record_steps else None
        self.workspace = torch.empty(max(16, dlm.lmhead_workspace_bytes(n, cfg.V, sample=sample_seed is not None, conf_mode=self.conf_mode)), dtype=torch.uint8, device=dev)
        self.attn_workspace = None    # sized per block (key split across workgroups)
        self._a_attn = self._a_lm = self._a_commit = None   # argument structs of a step, filled once per block
        self._sig = None
        # What a block's steps need besides the per-step pointers depends on the block index alone (the cache views,
        # the attention workspace size, the three argument structs): kept per block the first time the block is
        # visited, so that a rollout that comes back to a block (the next prompt of a batch job) pays that host work
        # once, not at every block boundary, where the GPU would sit idle meanwhile.
        self._plans = {}              # block -> dict(prefix, suffix, sig, a_attn, a_lm, a_commit)
        self._refresh_calls = {}      # (block, source pointers) -> prepared dlm_kv_refresh calls
        self._compact_args = None
        # optional hook(name, c_function, args_struct, stream_ptr, meta) -> return code, called INSTEAD of the plain
        # library call of a step or of a block's cache refresh (the benchmark's per-call event timing); None: the calls
        # go straight to the library
        self.on_call = None
        self.total_committed = torch.zeros(1, dtype=torch.int64, device=dev)
        self.block = -1
        self.step_idx = 0
        self.m_host = n          # host-side upper bound of the masked-row count
        self.diagnostics = True  # also write lse / zmax / z2nd (tests); the benchmark turns it off
        self._exact_rows = False
        # The polled row bound is one step old; the count itself is expected to be this fraction of it (a guess
        # that only selects which kernel shape is tried first; 0 turns the guess off).
        self.expect_ratio = 0.85
        self.late_bound = True    # False: the caller sets the row bound from the step just before (synchronous loop)
        # A step after which no sequence has more masked positions than the next step is certain to commit (1 with the
        # forced top-1 of the threshold rule, k with the top-k rule) tells the host that the NEXT step ends the block: a
        # loop that polls one step late then neither queues an empty step behind it nor waits for its result.
        self.predict_finish = True
        # ring of pinned host words: the commit kernel stores the total still-masked count straight into pinned
        # host memory, where the host watches for it (StepPoll)
        self._ring = [StepPoll() for _ in range(4)]
        self._ring_pos = 0
        self._last_poll = None

    def snapshot(self) -> dict:
        """Everything needed to resume this rollout elsewhere (another GpuRollout on the same workload, possibly in
        another process after a save): the token buffer, block mask, cache, the compacted row list with its count,
        both per-sequence count buffers and the host-side counters.  Synchronises the current stream."""
        torch.cuda.current_stream().synchronize()
        t = lambda x: None if x is None else x.clone()
        return dict(x=t(self.x), mask=t(self.mask), cache_k=t(self.cache_k), cache_v=t(self.cache_v),
                    row_idx=t(self.row_idx), m_dev=t(self.m_dev), remaining2=[t(r) for r in self._remaining2],
                    remaining_is=0 if self.remaining is self._remaining2[0] else 1, commit_step=t(self.commit_step),
                    block=self.block, step_idx=self.step_idx, m_host=self.m_host, exact_rows=self._exact_rows)

    def restore(self, snap: dict) -> None:
        """Continue from a snapshot() (taken at any step boundary of a block)."""
        for name in ("x", "mask", "cache_k", "cache_v", "row_idx", "m_dev"):
            getattr(self, name).copy_(snap[name])
        for dst, src in zip(self._remaining2, snap["remaining2"]):
            dst.copy_(src)
        self.remaining = self._remaining2[snap["remaining_is"]]
        if self.commit_step is not None and snap["commit_step"] is not None:
            self.commit_step.copy_(snap["commit_step"])
        self.block, self.step_idx = snap["block"], snap["step_idx"]
        self.m_host, self._exact_rows = snap["m_host"], snap["exact_rows"]
        if self.block >= 0:
            P, Lb, S = self.P, self.cfg.Lb, self.S
            self._prefix = (self.cache_k[:, :, :P], self.cache_v[:, :, :P], 0) if P > 0 else None
            self._suffix = (self.cache_k[:, :, P + Lb:P + Lb + S], self.cache_v[:, :, P + Lb:P + Lb + S], P + Lb) if S > 0 else None
            self._size_attn_workspace()
            self._a_attn = None

    def queue_poll(self) -> "StepPoll":
        """The StepPoll of the step queued last: its wait() returns the number of positions still masked after that
        step.  At most 3 polls may be outstanding (the slots are reused round-robin)."""
        return self._last_poll

    # geometry of the current block
    @property
    def P(self) -> int:
        return self.cfg.prompt + self.block * self.cfg.Lb

    @property
    def S(self) -> int:
        return self.cfg.L - self.P - self.cfg.Lb if self.cfg.dual_cache else 0

    def begin_block(self, block: int, init_mask: Optional[torch.Tensor] = None,
                    refresh_k: Optional[torch.Tensor] = None, refresh_v: Optional[torch.Tensor] = None) -> None:
        """Start denoising `block`: optionally refresh the cache from a full-sequence K/V image
        (prefix always, suffix too for the dual cache), reset the block mask, compact its rows."""
        cfg = self.cfg
        self.block, self.step_idx = block, 0
        P, Lb = self.P, cfg.Lb
        if refresh_k is not None:
            self._refresh(block, refresh_k, refresh_v)
        if init_mask is None:
            self.mask.fill_(1)
        else:
            self.mask.copy_(init_mask)
        if self.commit_step is not None:
            self.commit_step.fill_(-1)
        self._compact()
        self.m_host = cfg.B * Lb
        # fixed schedule: from a fully masked block the top-k rule leaves exactly Lb - k (s + 1) positions per
        # sequence after step s, so the LM-head launch can be sized exactly instead of from the late poll
        self._exact_rows = cfg.rule == "topk" and init_mask is None
        plan = self._plans.get(block)
        if plan is not None:
            self._prefix, self._suffix, self._sig = plan["prefix"], plan["suffix"], plan["sig"]
            self._a_attn, self._a_lm, self._a_commit = plan["a_attn"], plan["a_lm"], plan["a_commit"]
            return
        # the cache views of this block's prefix / suffix are the same for all of its steps
        S = self.S
        self._prefix = (self.cache_k[:, :, :P], self.cache_v[:, :, :P], 0) if P > 0 else None
        self._suffix = (self.cache_k[:, :, P + Lb:P + Lb + S], self.cache_v[:, :, P + Lb:P + Lb + S], P + Lb) if S > 0 else None
        self._size_attn_workspace()
        self._a_attn = None           # the step's argument structs are built at the block's first step

    def _refresh(self, block: int, refresh_k: torch.Tensor, refresh_v: torch.Tensor) -> None:
        """The block-boundary cache refresh: prefix rows always, suffix rows too for the dual cache.  The argument
        marshalling of the (at most two) dlm_kv_refresh calls is done once per (block, source image)."""
        cfg = self.cfg
        P, Lb = self.P, cfg.Lb
        key = (block, refresh_k.data_ptr(), refresh_v.data_ptr(), tuple(refresh_k.shape), refresh_k.stride(), refresh_v.stride())
        calls = self._refresh_calls.get(key)
        if calls is None:
            calls = []
            spans = ([(0, P)] if P > 0 else []) + ([(P + Lb, cfg.L)] if cfg.dual_cache and P + Lb < cfg.L else [])
            for lo, hi in spans:
                sk, sv = refresh_k[:, :, lo:hi], refresh_v[:, :, lo:hi]
                if hi > self.cache_k.shape[2] or self.cache_k.stride() != self.cache_v.stride():
                    raise ValueError("refresh image does not fit the cache")
                seg = dlm.kv_seg(sk, sv, 0)
                moved = 2 * 2 * cfg.B * cfg.Hkv * (hi - lo) * cfg.d * 2          # K and V, read + written
                calls.append((seg, (C.byref(seg), cfg.B, cfg.Hkv, cfg.d, self.cache_k.data_ptr(), self.cache_v.data_ptr(),
                                    self.cache_k.stride(0), self.cache_k.stride(1), self.cache_k.stride(2), lo), moved))
            if len(self._refresh_calls) > 4 * max(1, cfg.n_blocks):      # a caller that brings a new image every time
                self._refresh_calls.clear()
            self._refresh_calls[key] = calls
        sp = C.c_void_p(torch._C._cuda_getCurrentRawStream(self._dev_index))
        fn = dlm.lib().dlm_kv_refresh
        hook = self.on_call
        for _seg, args, moved in calls:
            # (the hook gets the positional arguments of dlm_kv_refresh without the stream, and calls fn(*args, stream))
            rc = fn(*args, sp) if hook is None else hook("kv_refresh", fn, args, sp, dict(bytes=moved))
            if rc:
                raise dlm.DlmError(rc, dlm.last_error())

    def _compact(self) -> None:
        """dlm_mask_compact of the block mask into the row list (arguments marshalled once)."""
        if self._compact_args is None:
            self._compact_args = (self.mask.data_ptr(), self.mask.stride(0), self.cfg.B, self.cfg.Lb,
                                  self.row_idx.data_ptr(), self.m_dev.data_ptr())
        rc = dlm.lib().dlm_mask_compact(*self._compact_args, C.c_void_p(torch._C._cuda_getCurrentRawStream(self._dev_index)))
        if rc:
            raise dlm.DlmError(rc, dlm.last_error())

    def _size_attn_workspace(self) -> None:
        """The attention call may split the keys across workgroups when it is given a workspace; its size depends on
        the block's key count, so it is queried (and the buffer grown) once per block, never inside a step."""
        cfg, Lb = self.cfg, self.cfg.Lb
        blk = (self.cache_k[:, :, :Lb], self.cache_v[:, :, :Lb], self.P)      # stands in for the step's block K/V (same shape)
        need = dlm.block_attn_workspace_bytes(self.O, prefix=self._prefix, block=blk, suffix=self._suffix,
                                              mask_mode=_MASKS[cfg.mask_mode], block_size=cfg.bs, q_pos0=self.P)
        if need > (0 if self.attn_workspace is None else self.attn_workspace.numel()):
            self.attn_workspace = torch.empty(need, dtype=torch.uint8, device=self.dev)
            self._plans.clear()       # the structs kept for other blocks point at the old workspace

    def _prepare_step(self, q, kblk, vblk, hidden) -> None:
        """Fill the three argument structs of a denoising step once per block (all validation happens here); the steps
        of the block then only exchange the pointers and counters that change from step to step."""
        cfg = self.cfg
        P, Lb = self.P, cfg.Lb
        diag = self.diagnostics
        self._sig = (q.shape, q.stride(), kblk.shape, kblk.stride(), vblk.stride(), hidden.shape, hidden.stride(), diag)
        self._a_attn = dlm._attn_args(q, self.O, self._prefix, (kblk, vblk, P), self._suffix,
                                      mask_mode=_MASKS[cfg.mask_mode], block_size=cfg.bs, q_pos0=P,
                                      lse=self.lse_attn if diag else None, seq_active=self.remaining,
                                      workspace=self.attn_workspace)
        self._a_lm = dlm._lmhead_args(hidden.view(cfg.B * Lb, cfg.Dh), self.w, self.conf, self.tok,
                                      M=self.m_host, row_idx=self.row_idx, m_dev=self.m_dev,
                                      forbid_token=cfg.forbid_token, out_scatter=True,
                                      lse=self.lse if diag else None, zmax=self.zmax if diag else None,
                                      z2nd=self.z2nd if diag else None, workspace=self.workspace,
                                      inv_temperature=self.inv_temperature, sample_seed=self.sample_seed,
                                      sample_step=0, sample_stream=self.sample_stream, conf_mode=self.conf_mode)
        self._a_commit = dlm._commit_args(self.conf, self.tok, self.x, self.mask, self.n_commit, self.remaining,
                                          x_pos0=P, rule=_RULES[cfg.rule], threshold=cfg.tau, force_top1=True, k=cfg.k,
                                          commit_now=self.commit_now, next_row_idx=self.row_idx, next_m=self.m_dev,
                                          commit_step=self.commit_step, step=0, writeback=dlm.WB_WHILE_ACTIVE,
                                          active_in=self.remaining, src_block=(kblk, vblk, 0),
                                          cache_k=self.cache_k, cache_v=self.cache_v, cache_pos0=P,
                                          host_remaining_total=self._ring[0].word, host_remaining_max=self._ring[0].word_max)
        self._rem_ptr = [r.data_ptr() for r in self._remaining2]
        self._ring_ptr = [sp.ptr for sp in self._ring]
        self._ring_ptr_max = [sp.ptr_max for sp in self._ring]
        self._lib = dlm.lib()
        self._plans[self.block] = dict(prefix=self._prefix, suffix=self._suffix, sig=self._sig, a_attn=self._a_attn,
                                       a_lm=self._a_lm, a_commit=self._a_commit)   # per-step pointers are rewritten by step()

    def step(self, q: torch.Tensor, kblk: torch.Tensor, vblk: torch.Tensor, hidden: torch.Tensor) -> None:
        """Enqueue one denoising step.  q [B, Lb, Hq, d]; kblk, vblk [B, Hkv, Lb, d]; hidden [B, Lb, Dh].

        Every step of a block passes tensors of one shape and layout (checked); what differs between steps is a handful
        of pointers and counters, so the argument structs are filled once per block (_prepare_step) and only those
        fields are rewritten here: the host side of a step is three foreign calls."""
        cfg = self.cfg
        Lb = cfg.Lb
        if self._a_attn is None or self._sig != (q.shape, q.stride(), kblk.shape, kblk.stride(), vblk.stride(),
                                                 hidden.shape, hidden.stride(), self.diagnostics):
            self._prepare_step(q, kblk, vblk, hidden)
        for t in (q, kblk, vblk, hidden):
            if not t.is_cuda or t.dtype != torch.bfloat16:
                raise ValueError("step inputs must be bf16 tensors on the GPU")
        pos = self._ring_pos
        poll = self._ring[pos]
        self._ring_pos = (pos + 1) % len(self._ring)
        poll.arm()                           # before anything of this step is queued
        # the raw handle of torch's current stream on this device, looked up once per step (the Stream object that
        # torch.cuda.current_stream() builds costs several microseconds of Python)
        sp = C.c_void_p(torch._C._cuda_getCurrentRawStream(self._dev_index))
        if self._exact_rows:
            self.m_host = max(1, cfg.B * max(Lb - cfg.k * self.step_idx, 0))
        first = self.step_idx == 0
        L = self._lib
        kp, vp = kblk.data_ptr(), vblk.data_ptr()
        # 1. attention; from a block's second step on, sequences with nothing left masked after the previous step are
        #    skipped: the LM head reads only masked rows, so nothing would consume their attention output
        a = self._a_attn
        a.q = q.data_ptr()
        a.block.k, a.block.v = kp, vp
        idx_prev = 0 if self.remaining is self._remaining2[0] else 1
        a.seq_active = None if first else self._rem_ptr[idx_prev]
        hook = self.on_call
        rc = L.dlm_block_attn(C.byref(a), sp) if hook is None else hook("block_attn", L.dlm_block_attn, a, sp, dict(first=first))
        if rc:
            raise dlm.DlmError(rc, dlm.last_error())
        # 2. LM head on the still-masked rows (count read on the device; the host's bound sizes the launch)
        a = self._a_lm
        a.hidden = hidden.data_ptr()
        a.M = self.m_host
        a.M_expected = 0 if (self._exact_rows or not self.late_bound) else int(self.m_host * self.expect_ratio)
        a.sample_step = ((self.block << 16) | self.step_idx) & 0xFFFFFFFF
        rc = L.dlm_lmhead_confidence(C.byref(a), sp) if hook is None else hook("lmhead_confidence", L.dlm_lmhead_confidence, a, sp, None)
        if rc:
            raise dlm.DlmError(rc, dlm.last_error())
        # 3. selection, commit, compaction and the cache write-back of the block's K/V.  First step of a block: a
        #    sequence that finishes right away is copied by a launch of its own.  Later steps: every sequence that was
        #    still masked after the previous step is copied inside the selection's launch (the last such copy is its
        #    final step's K/V: the same cache contents, one launch fewer per step).
        idx_new = self.step_idx & 1
        a = self._a_commit
        a.remaining = self._rem_ptr[idx_new]
        a.step = self.step_idx
        a.writeback = dlm.WB_BLOCK_WHEN_DONE if first else dlm.WB_WHILE_ACTIVE
        a.active_in = None if first else self._rem_ptr[idx_prev]
        a.src_block.k, a.src_block.v = kp, vp
        a.host_remaining_total = self._ring_ptr[pos]
        a.host_remaining_max = self._ring_ptr_max[pos]
        rc = L.dlm_unmask_commit(C.byref(a), sp) if hook is None else hook("unmask_commit", L.dlm_unmask_commit, a, sp, dict(first=first, remaining=self._remaining2[idx_new]))
        if rc:
            raise dlm.DlmError(rc, dlm.last_error())
        self.remaining = self._remaining2[idx_new]
        self._last_poll = poll
        self.step_idx += 1

    def next_step_finishes(self, poll: "StepPoll") -> bool:
        """poll: a waited-for StepPoll of this block.  True when the step AFTER the polled one is certain to leave nothing
        masked: every sequence has at most as many masked positions left as the rule commits per step."""
        if not self.predict_finish:
            return False
        return poll.left_max <= (self.cfg.k if self.cfg.rule == "topk" else 1)

    def set_row_bound(self, m: int) -> None:
        """Tell the driver an upper bound of the masked-row count (sizes the LM-head launch)."""
        if not self._exact_rows:
            self.m_host = max(1, min(int(m), self.cfg.B * self.cfg.Lb))

    def run_block(self, block: int, inputs: Callable[[int, int], tuple], init_mask=None,
                  refresh=None, lagged: bool = True, max_steps: Optional[int] = None) -> dict:
        """Denoise one block to completion.  inputs(block, step) -> (q, kblk, vblk, hidden) on the GPU.

        Returns {"steps": queued steps, "empty": queued steps that found nothing masked}.
        With lagged=False the host waits for every step's `remaining` before queuing the next.
        """
        cfg = self.cfg
        rk, rv = refresh if refresh is not None else (None, None)
        self.late_bound = lagged
        self.begin_block(block, init_mask, rk, rv)
        max_steps = cfg.Lb + 1 if max_steps is None else max_steps
        pending = []   # StepPoll of the steps already queued
        steps = empty = 0
        done = False
        while not done and steps < max_steps:
            self.step(*inputs(block, steps))
            steps += 1
            pending.append(self.queue_poll())
            # look at the newest result that is allowed to be waited for
            lag = 1 if lagged else 0
            while len(pending) > lag:
                p0 = pending.pop(0)
                rem = p0.wait()
                self.set_row_bound(rem if rem > 0 else 1)
                if rem == 0:
                    done = True
                    empty = len(pending)   # steps queued after the finishing one found nothing to do
                    pending.clear()
                    break
                if len(pending) == 1 and self.next_step_finishes(p0):
                    done = True            # the step already queued behind the polled one ends the block: no need to wait
                    pending.clear()
                    break
        if not done:
            for p0 in pending:
                if p0.wait() == 0:
                    done = True
            if not done:
                raise RuntimeError(f"block {block} not finished after {steps} steps")
        return {"steps": steps - empty, "empty": empty}


class StepRunner:
    """Runs an exact number of productive denoising steps, continuing across blocks and restarting
    the rollout after its last block.  Used by the benchmark and by long-running callers.

    setup(block) -> dict(init_mask=None | tensor, refresh=None | (k, v), restart=bool) describes how a
    block starts; inputs(block, step) -> (q, kblk, vblk, hidden).  A step is productive when it found
    masked positions; with the one-step-late poll at most one queued step per block is not.
    """

    def __init__(self, g: GpuRollout, inputs: Callable[[int, int], tuple], setup: Callable[[int], dict],
                 on_restart: Optional[Callable[[], None]] = None, lagged: bool = True, on_step=None):
        self.g, self.inputs, self.setup, self.on_restart, self.lagged = g, inputs, setup, on_restart, lagged
        g.late_bound = lagged
        self.on_step = on_step          # optional hook(g, fn) wrapping the enqueue of one step (timing)
        self.block = -1
        self.in_block = False
        self.queued = 0                 # steps queued in the current block
        self.known = 0                  # of those, how many are known to be productive
        self.rem_prev = 0               # masked count before the oldest not-yet-polled step
        self.pending = []               # StepPoll of the steps queued and not yet polled
        self.committed = 0
        self.empty = 0
        self.blocks_done = 0
        self.steps_per_block = []
        self.log = []                   # per polled step, in queue order: (block, masked before, masked after)

    def _begin_next_block(self):
        g = self.g
        self.block = (self.block + 1) % g.cfg.n_blocks
        if self.block == 0 and self.on_restart is not None:
            self.on_restart()
        st = self.setup(self.block)
        rk, rv = st.get("refresh") or (None, None)
        g.begin_block(self.block, st.get("init_mask"), rk, rv)
        self.in_block, self.queued, self.known = True, 0, 0
        self.rem_prev = int(st.get("n_masked", g.cfg.B * g.cfg.Lb))
        self.pending = []

    def _poll_one(self) -> bool:
        """Wait for the oldest queued step's result; returns True when it finished the block."""
        self._polled = self.pending.pop(0)
        rem = self._polled.wait()
        self.log.append((self.block, self.rem_prev, rem))
        if self.rem_prev > 0:
            self.known += 1
            self.committed += self.rem_prev - rem
        else:
            self.empty += 1
        self.rem_prev = rem
        self.g.set_row_bound(rem if rem > 0 else 1)
        return rem == 0

    def run(self, n_steps: int) -> dict:
        g = self.g
        done_steps = 0                  # productive steps completed and polled in this call
        start_committed, start_empty = self.committed, self.empty
        while done_steps < n_steps:
            if not self.in_block:
                self._begin_next_block()
            unpolled = len(self.pending)
            # queue one more step unless every step we still need might already be in flight
            if done_steps + unpolled < n_steps:
                args = self.inputs(self.block, self.queued)
                if self.on_step is not None:
                    self.on_step(g, lambda: g.step(*args))
                else:
                    g.step(*args)
                self.queued += 1
                self.pending.append(g.queue_poll())
            lag = 1 if (self.lagged and done_steps + len(self.pending) < n_steps) else 0
            while len(self.pending) > lag:
                was_productive = self.rem_prev > 0
                finished = self._poll_one()
                if was_productive:
                    done_steps += 1
                if not finished and len(self.pending) == 1 and g.next_step_finishes(self._polled):
                    # the one step queued behind the polled one commits everything that is left: it is accounted for
                    # without being waited for, and the next block's work is queued right behind it
                    self.pending.pop(0)
                    self.log.append((self.block, self.rem_prev, 0))
                    self.known += 1
                    self.committed += self.rem_prev
                    self.rem_prev = 0
                    done_steps += 1
                    finished = True
                if finished:
                    # whatever is still queued in this block found nothing masked
                    while self.pending:
                        self._poll_one()
                    self.steps_per_block.append(self.known)
                    self.blocks_done += 1
                    self.in_block = False
                    break
        return dict(steps=done_steps, committed=self.committed - start_committed,
                    empty=self.empty - start_empty)
