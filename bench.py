#!/usr/bin/env python3
"""Benchmark of the rollout denoising step on one MI355X.

A "step" is one denoising step of the LLaDA-8B-shaped rollout (batch 8, 32 heads, head_dim 128,
hidden 4096, vocabulary 126464, prompt 512, 256 generated tokens in 8 blocks of 32, threshold 0.9
with the most confident position always committed, prefix cache refreshed at every block start):
block attention against [prefix | block], LM head -> confidence on the still-masked rows,
threshold commit with KV write-back, plus the block-boundary cache refresh when a block starts.
Steps continue across blocks and rollouts; K productive steps are timed.

Prints ONE JSON line: committed tokens/s, the roofline of the dominant kernel (the LM head, which
streams the 1.04 GB W_vocab every step) measured with HIP events on the launch stream, and the CPU
oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM bytes per LM-head launch on the default workload, from two rocprofv3 --pmc runs (FETCH_SIZE x 2.0,
# WRITE_SIZE x 1.0, factors calibrated with a 1 GiB copy); summary and commands in
# profiles/lmhead_c2_rollout_hbm_traffic.md.  Only valid for --config c2.
LMHEAD_C2_TRAFFIC_BYTES = 1097.2e6


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1500)
    ap.add_argument("--warmup", type=int, default=150)
    ap.add_argument("--config", default="c2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true", help="skip per-step LM-head event timing")
    ap.add_argument("--sync-loop", action="store_true", help="poll every step synchronously (no one-step-late poll)")
    ap.add_argument("--expect-ratio", type=float, default=None,
                    help="the driver's guess of (rows in a step) / (late row bound); 0 = no guess; default: the driver's")
    ap.add_argument("--set-option", action="append", default=[], metavar="NAME=VALUE",
                    help="library tuning knob (dlm_set_option) applied before the run; may be repeated")
    ap.add_argument("--dump-steps", default=None, metavar="FILE",
                    help="write one line per timed step: block, rows masked before / after, row bound, LM-head us")
    ap.add_argument("--kernel", default=None, choices=["lmhead", "attn_fullseq", "fullpass"],
                    help="time ONE kernel on random inputs instead of the rollout (record only, for profiles): "
                         "lmhead = dlm_lmhead_confidence at --rows rows on the config's W shape; attn_fullseq = "
                         "dlm_block_attn (and, with --backward, dlm_block_attn_bwd) on 64 x 4096 tokens, 32/8 heads, d = 128; "
                         "fullpass = one full-sequence block-diffusion pass of workload c5b (attention, row compaction, "
                         "LM head on the masked rows, one commit per block of 4), each part timed")
    ap.add_argument("--rows", type=int, default=8192, help="--kernel lmhead: number of hidden rows M")
    ap.add_argument("--lmhead-variant", default="-1", help="--kernel lmhead: comma-separated entries of the shape table (-1 = planner)")
    ap.add_argument("--zeros", action="store_true", help="--kernel lmhead: all-zero operands (no data-dependent power)")
    ap.add_argument("--mask", default="block_causal", choices=["full", "block_causal"], help="--kernel attn_fullseq")
    ap.add_argument("--batch", type=int, default=64, help="--kernel attn_fullseq: sequences")
    ap.add_argument("--backward", action="store_true", help="--kernel attn_fullseq: also time the backward pass")
    ap.add_argument("--reps", type=int, default=3, help="--kernel: timed calls per measurement")
    return ap.parse_args()


def micro(args):
    """One kernel on random inputs (normal bf16 values, the rollout's W scale): a JSON line per measurement."""
    import torch
    from paper_2604_04215_amd import binding as dlm
    from paper_2604_04215_amd import synth
    dlm.lib()
    dev = "cuda:0"
    torch.manual_seed(0)

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    if args.kernel == "lmhead":
        cfg = synth.CONFIGS[args.config]
        M, V, Dh = args.rows, cfg.V, cfg.Dh
        if args.zeros:
            w = torch.zeros((V, Dh), device=dev, dtype=torch.bfloat16)
            h = torch.zeros((M, Dh), device=dev, dtype=torch.bfloat16)
        else:
            w = (torch.randn((V, Dh), device=dev) * Dh ** -0.25).bfloat16()
            h = torch.randn((M, Dh), device=dev).bfloat16()
        conf = torch.empty(M, device=dev)
        tok = torch.empty(M, dtype=torch.int32, device=dev)
        ws = torch.empty(dlm.lmhead_workspace_bytes(M, V), dtype=torch.uint8, device=dev)
        for variant in [int(x) for x in args.lmhead_variant.split(",")]:
            dlm.set_option("lmhead_variant", variant)
            ms = timed(lambda: dlm.lmhead_confidence(h, w, conf, tok, workspace=ws, forbid_token=V - 1), args.reps)
            print(json.dumps({"kernel": "dlm_lmhead_confidence", "M": M, "V": V, "Dh": Dh, "variant": variant,
                              "data": "zeros" if args.zeros else "normal", "us": round(ms * 1e3, 1),
                              "tflops": round(2.0 * M * V * Dh / ms / 1e9, 1),
                              "w_stream_gbs": round(V * Dh * 2 / ms / 1e6, 1)}), flush=True)
        dlm.set_option("lmhead_variant", -1)
        return
    if args.kernel == "fullpass":
        cfg = synth.FULLPASS["c5b"]
        B, L = cfg.B, cfg.L
        rb = lambda *shape, std=1.0: (torch.randn(*shape, device=dev) * std).to(torch.bfloat16)
        w = rb(cfg.V, cfg.Dh, std=cfg.Dh ** -0.25)
        q, k, v = rb(B, L, cfg.Hq, cfg.d), rb(B, cfg.Hkv, L, cfg.d), rb(B, cfg.Hkv, L, cfg.d)
        hid = rb(B * L, cfg.Dh)
        out = torch.empty_like(q)
        mask0 = (torch.rand(B, L, device=dev) < 0.5).to(torch.uint8)     # Bernoulli(0.5) masking
        mask = mask0.clone()
        row_idx = torch.zeros(B * L, dtype=torch.int32, device=dev)
        m_dev = torch.zeros(1, dtype=torch.int32, device=dev)
        dlm.mask_compact(mask, row_idx, m_dev)
        torch.cuda.synchronize()
        M = int(m_dev.item())
        conf = torch.zeros(B, L, device=dev)
        tok = torch.zeros(B, L, dtype=torch.int32, device=dev)
        x = torch.zeros(B, L, dtype=torch.int32, device=dev)
        n_commit = torch.zeros(B, dtype=torch.int32, device=dev)
        remaining = torch.zeros(B, dtype=torch.int32, device=dev)
        ws = torch.empty(dlm.lmhead_workspace_bytes(M, cfg.V), dtype=torch.uint8, device=dev)
        pairs = (L // cfg.bs) * (L // cfg.bs + 1) // 2 * cfg.bs * cfg.bs

        def commit():
            mask.copy_(mask0)
            dlm.unmask_commit(conf, tok, x, mask, n_commit, remaining, x_pos0=0, group_len=cfg.bs,
                              rule=dlm.RULE_THRESHOLD, threshold=cfg.tau)

        parts = [("dlm_block_attn", lambda: dlm.block_attn(q, out, block=(k, v, 0), mask_mode=dlm.MASK_BLOCK_CAUSAL,
                                                            block_size=cfg.bs, q_pos0=0), 4.0 * B * cfg.Hq * cfg.d * pairs),
                 ("dlm_mask_compact", lambda: dlm.mask_compact(mask0, row_idx, m_dev), 0.0),
                 ("dlm_lmhead_confidence", lambda: dlm.lmhead_confidence(hid, w, conf, tok, row_idx=row_idx, M=M,
                                                                         forbid_token=cfg.V - 1, out_scatter=True,
                                                                         workspace=ws), 2.0 * M * cfg.V * cfg.Dh),
                 ("dlm_unmask_commit (incl. a mask reset copy)", commit, 0.0)]
        total = 0.0
        for name, fn, flop in parts:
            ms = timed(fn, args.reps)
            total += ms
            rec = {"kernel": name, "workload": "c5b full pass", "ms": round(ms, 3)}
            if flop:
                rec["tflops"] = round(flop / ms / 1e9, 1)
            if name == "dlm_lmhead_confidence":
                rec["M"] = M
            print(json.dumps(rec), flush=True)
        print(json.dumps({"kernel": "whole pass", "workload": "c5b full pass", "ms": round(total, 2),
                          "positions": B * L, "masked": M}), flush=True)
        return
    B, L, Hq, Hkv, d, bs = args.batch, 4096, 32, 8, 128, 4
    mk = lambda *shape: torch.randn(shape, device=dev).bfloat16()
    q, do, k, v = mk(B, L, Hq, d), mk(B, L, Hq, d), mk(B, Hkv, L, d), mk(B, Hkv, L, d)
    out = torch.empty_like(q)
    lse = torch.empty((B, Hq, L), dtype=torch.float32, device=dev)
    mode = dlm.MASK_FULL if args.mask == "full" else dlm.MASK_BLOCK_CAUSAL
    pairs = L * L if args.mask == "full" else L * (L + bs) / 2
    ms = timed(lambda: dlm.block_attn(q, out, block=(k, v, 0), mask_mode=mode, block_size=bs, lse=lse), args.reps)
    print(json.dumps({"kernel": "dlm_block_attn", "mask": args.mask, "B": B, "L": L, "heads": [Hq, Hkv], "d": d,
                      "ms": round(ms, 3), "tflops": round(4.0 * B * Hq * d * pairs / ms / 1e9, 1)}), flush=True)
    if args.backward:
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        ws = torch.empty(dlm.block_attn_bwd_workspace_bytes(B * L, Hq), dtype=torch.uint8, device=dev)
        ms = timed(lambda: dlm.block_attn_bwd(q, out, do, lse, dq, block=(k, v, 0), d_block=(dk, dv), mask_mode=mode,
                                              block_size=bs, workspace=ws), args.reps)
        print(json.dumps({"kernel": "dlm_block_attn_bwd", "mask": args.mask, "B": B, "L": L, "heads": [Hq, Hkv], "d": d,
                          "ms": round(ms, 3), "tflops": round(10.0 * B * Hq * d * pairs / ms / 1e9, 1)}), flush=True)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (sequences are independent, so a multi-GPU "
              "rollout is N copies of this program with B/N sequences each); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2604_04215_amd import binding as dlm
    from paper_2604_04215_amd import synth
    from paper_2604_04215_amd.rollout import GpuRollout, StepRunner

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dlm.lib()  # fail loudly if the HIP library is missing
    for kv in args.set_option:
        name, _, val = kv.partition("=")
        dlm.set_option(name, int(val))
    if args.kernel:
        micro(args)
        return
    dev = "cuda:0"
    cfg = synth.CONFIGS[args.config]
    t_setup = time.time()

    def to_dev(u16):
        return torch.from_numpy(np.ascontiguousarray(u16).view(np.int16)).view(torch.bfloat16).to(dev)

    w_host = synth.w_vocab(cfg)
    w = to_dev(w_host)
    g = GpuRollout(cfg, w, dev)
    g.diagnostics = False
    if args.expect_ratio is not None:
        g.expect_ratio = args.expect_ratio
    x0 = torch.from_numpy(synth.initial_tokens(cfg, cfg.L)).to(dev)
    images = {}

    def image(block):
        if block not in images:
            k, v = synth.cache_kv(cfg, block)
            images[block] = (to_dev(k), to_dev(v))
        return images[block]

    init_host = {b: synth.initial_block_mask(cfg, b) for b in range(cfg.n_blocks)}
    init_masks = {b: torch.from_numpy(m).to(dev) for b, m in init_host.items()}
    n_masked0 = {b: int(m.sum()) for b, m in init_host.items()}      # known on the host: no device reduction per block
    pool = {}

    def inputs(block, step):
        key = (block, step)
        if key not in pool:
            kb, vb = synth.step_kv(cfg, block, step)
            pool[key] = (to_dev(synth.step_q(cfg, block, step)), to_dev(kb), to_dev(vb),
                         to_dev(synth.step_hidden(cfg, block, step)))
        return pool[key]

    def setup(block):
        # block 0 installs the prompt cache image; later blocks refresh it when the workload says so
        refresh = image(block) if (block == 0 or cfg.refresh) else None
        # a block that starts fully masked is announced as such (no mask tensor): the driver then knows the top-k
        # rule's row schedule exactly
        full = n_masked0[block] == cfg.B * cfg.Lb
        return dict(init_mask=None if full else init_masks[block], refresh=refresh, n_masked=n_masked0[block])

    def restart():
        g.x.copy_(x0)

    # ---- discovery pass (untimed): generates and uploads every step input the rollout touches ------
    runner = StepRunner(g, inputs, setup, on_restart=restart, lagged=not args.sync_loop)
    while runner.blocks_done < cfg.n_blocks:
        runner.run(1)
    # make sure the extra step a one-step-late poll may queue after a block's last step exists too
    steps_per_block = list(runner.steps_per_block[:cfg.n_blocks])
    for b, s in enumerate(steps_per_block):
        inputs(b, s)
    while runner.in_block:        # finish the block the discovery loop may have started
        runner.run(1)
    torch.cuda.synchronize()
    rollout_steps = sum(steps_per_block)
    setup_s = time.time() - t_setup

    # ---- LM-head event timing hook ------------------------------------------------------------------
    lm_events = []
    orig_lmhead = dlm.lmhead_confidence

    def timed_lmhead(*a, **kw):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(torch.cuda.current_stream())
        orig_lmhead(*a, **kw)
        e1.record(torch.cuda.current_stream())
        lm_events.append((e0, e1, kw.get("M")))

    import paper_2604_04215_amd.rollout as ro_mod

    # ---- warm-up, then the timed region -------------------------------------------------------------
    runner.run(args.warmup) if args.warmup > 0 else None
    torch.cuda.synchronize()
    if not args.no_kernel_events:
        ro_mod.dlm.lmhead_confidence = timed_lmhead
    c0, e0, log0 = runner.committed, runner.empty, len(runner.log)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    res = runner.run(args.steps)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ro_mod.dlm.lmhead_confidence = orig_lmhead
    elapsed = t1 - t0
    committed = runner.committed - c0
    empty = runner.empty - e0
    assert res["steps"] == args.steps

    # ---- roofline of the LM head (dominant kernel): algorithmic bytes / measured duration -----------
    # One dlm_lmhead_confidence call streams W_vocab once (V*Dh*2 bytes), gathers M hidden rows
    # (M*Dh*2 bytes) and writes a handful of bytes per row; M is the number of rows masked before the step.
    roof = None
    w_bytes = cfg.V * cfg.Dh * 2
    if lm_events:
        log = runner.log[log0:]
        assert len(log) == len(lm_events)
        ms, rows = [], []
        for (a, b, _bound), (_, before, _after) in zip(lm_events, log):
            if before > 0:                      # launches that found nothing masked move no data
                ms.append(a.elapsed_time(b))
                rows.append(before)
        if args.dump_steps:                     # per step: rows masked before, host-side row bound, LM-head call in us
            with open(args.dump_steps, "w") as f:
                for (a, b, bound), (blk, before, after) in zip(lm_events, log):
                    f.write(f"{blk} {before} {after} {bound} {a.elapsed_time(b) * 1e3:.1f}\n")
        avg_ms = sum(ms) / len(ms)
        mean_rows = sum(rows) / len(rows)
        bytes_per_launch = w_bytes + mean_rows * cfg.Dh * 2 + mean_rows * 8
        achieved = bytes_per_launch / (avg_ms * 1e-3) / 1e9
        roof = dict(bound="hbm", achieved=round(achieved, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(achieved / HBM_PEAK_GBS, 4),
                    traffic=int(LMHEAD_C2_TRAFFIC_BYTES) if args.config == "c2" else None,
                    kernel="lmhead_kernel (M <= 192) or lmhead_pair_kernel (above) + lmhead_reduce_kernel (one dlm_lmhead_confidence call)",
                    avg_us=round(avg_ms * 1e3, 2), median_us=round(sorted(ms)[len(ms) // 2] * 1e3, 2),
                    launches=len(ms), bytes_per_launch=int(bytes_per_launch), mean_rows=round(mean_rows, 1),
                    flops_per_launch=int(2 * mean_rows * cfg.Dh * cfg.V),
                    mfma_tflops=round(2 * mean_rows * cfg.Dh * cfg.V / (avg_ms * 1e-3) / 1e12, 1))

    # ---- CPU oracle on a bounded sample of the same workload ----------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        tc0 = time.perf_counter()
        n_tok = n_steps_cpu = n_seq = 0
        for b in range(cfg.B):                       # whole sequences of block 0 until ~12 s of CPU work
            o = oracle.OracleRollout(cfg, synth, seqs=[b], w=w_host)
            o.begin_block(0)
            while o.mask.any():
                r = o.step()
                n_tok += int(r["n_commit"].sum())
                n_steps_cpu += 1
            n_seq += 1
            if time.perf_counter() - tc0 > 12.0:
                break
        tc = time.perf_counter() - tc0
        cpu = dict(value=round(n_tok / tc, 3), unit="committed tokens/s", cores=oracle.num_threads(), kind="oracle",
                   sample=f"sequences 0..{n_seq - 1} of the batch, one at a time, block 0 (prefix {cfg.prompt} + block "
                          f"{cfg.Lb}) to completion: {n_steps_cpu} denoising steps, {n_tok} tokens committed in {tc:.1f} s")

    out = {
        "metric": "committed tokens/sec per denoise step",
        "value": round(committed / elapsed, 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(elapsed / args.steps * 1e3, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "c2: LLaDA-8B-shaped rollout, B=8, 32 heads MHA, d=128, hidden 4096, V=126464, "
                               "prompt 512, gen 256 in 8 blocks of 32, threshold 0.9 + forced top-1, "
                               "prefix cache refreshed per block" if args.config == "c2" else args.config,
                   "committed_tokens": committed, "tokens_per_step": round(committed / args.steps, 3),
                   "steps_per_rollout": rollout_steps, "steps_per_block": steps_per_block,
                   "empty_steps_in_timed_region": empty,
                   "loop": "sync" if args.sync_loop else "one-step-late poll", "setup_s": round(setup_s, 1)},
        "roofline": roof,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
