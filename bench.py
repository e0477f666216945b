#!/usr/bin/env python3
"""Benchmark of the rollout denoising step on one MI355X.

A "step" is one denoising step of the LLaDA-8B-shaped rollout (batch 8, 32 heads, head_dim 128,
hidden 4096, vocabulary 126464, prompt 512, 256 generated tokens in 8 blocks of 32, threshold 0.9
with the most confident position always committed, prefix cache refreshed at every block start):
block attention against [prefix | block], LM head -> confidence on the still-masked rows,
threshold commit with KV write-back, plus the block-boundary cache refresh when a block starts.
Steps continue across blocks and rollouts; K productive steps are timed, with nothing but the step's
own launches inside the timed region.

After the timed region a separate pass of a FIXED number of steps (--sample-steps, independent of
--steps) brackets every library call with HIP events on the launch stream; from it come the per-call
durations, the algorithmic bytes / FLOP of each call (from the row and sequence counts the device
reported for that very step) and the fraction of the roof that binds each of them.

Prints ONE JSON line: committed tokens/s; `roofline` for the call that takes most of the step; `kernels`
with the same figures for dlm_block_attn, dlm_lmhead_confidence, dlm_unmask_commit and dlm_kv_refresh,
against nominal and measured peaks; `cpu_baseline`: the CPU oracle timed on a bounded sample of the
same workload, with its linear extrapolation to the whole batch.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, nominal
MFMA_PEAK_TFLOPS = 2500.0      # dense bf16 MFMA, nominal
RIDGE = MFMA_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)     # FLOP per byte at which the two roofs meet (312.5)
# HBM bytes per LM-head launch on the default workload, from two rocprofv3 --pmc runs (FETCH_SIZE x 2.0,
# WRITE_SIZE x 1.0, factors calibrated with a 1 GiB copy); summary and commands in
# profiles/lmhead_c2_rollout_hbm_traffic.md.  Only valid for --config c2 with the default W distribution.
LMHEAD_C2_TRAFFIC_BYTES = 1045.1e6

WORKLOADS = {
    "c1": "c1: tiny single block, B=1, 4 heads MHA, d=64, hidden 256, V=2048, prefix 256, block 32 with 16 masked, "
          "threshold 0.9 + forced top-1",
    "c2": "c2: LLaDA-8B-shaped rollout, B=8, 32 heads MHA, d=128, hidden 4096, V=126464, prompt 512, gen 256 in 8 blocks "
          "of 32, threshold 0.9 + forced top-1, prefix cache refreshed per block",
    "c3": "c3: dual-cache rollout, B=16, 32 heads MHA, d=128, hidden 4096, V=126464, prompt 1024, gen 512 in 16 blocks of "
          "32, keys = prefix + block + suffix (1536), threshold 0.9 + forced top-1, caches refreshed per block",
    "c4": "c4: Dream-7B-shaped GQA rollout, B=32, 28 query / 4 KV heads, d=128, hidden 3584, V=152064, prompt 768, gen 256 "
          "in 8 blocks of 32, fixed top-k=4 commits per step",
    "c5a": "c5a: block-diffusion rollout of the last block, B=64, 32 query / 8 KV heads, d=128, hidden 4096, V=157184, "
           "block-causal with block size 4 against a 4092-token cache, threshold 0.95 + forced top-1",
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1500)
    ap.add_argument("--warmup", type=int, default=150)
    ap.add_argument("--config", default="c2", choices=sorted(WORKLOADS))
    ap.add_argument("--w-dist", default="var", choices=["var", "std"],
                    help="W_vocab ~ N(0, x) with x = Dh^-1/2 read as a variance (default: logit std Dh^1/4, both branches of the "
                         "threshold rule fire) or as a standard deviation (logit std 1: the threshold never fires and every "
                         "step commits exactly one position per sequence)")
    ap.add_argument("--ramp-steps", type=int, default=300,
                    help="untimed steps queued before the --warmup steps so that a short run is timed at the same clock "
                         "as a long one (the discovery pass before them leaves the GPU mostly idle)")
    ap.add_argument("--ramp-seconds", type=float, default=0.4,
                    help="the untimed ramp lasts at least this long (more --ramp-steps are queued until it has): a workload of "
                         "small launches (c1: 20 us of kernels per step) brings the clock up far more slowly than one that "
                         "streams a gigabyte per step, and runs at half its steady rate for the first ~0.1 s")
    ap.add_argument("--sample-steps", type=int, default=400,
                    help="steps of the per-call event-timing pass that follows the timed region (0 = skip it)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--oracle-seqs", type=int, default=0,
                    help="cpu_baseline: sequences the oracle runs (block 0 to completion); 0 = as many as fit in ~12 s")
    ap.add_argument("--no-peaks", action="store_true", help="skip the achievable-peak micro-benchmarks")
    ap.add_argument("--sync-loop", action="store_true", help="poll every step synchronously (no one-step-late poll)")
    ap.add_argument("--expect-ratio", type=float, default=None,
                    help="the driver's guess of (rows in a step) / (late row bound); 0 = no guess; default: the driver's")
    ap.add_argument("--set-option", action="append", default=[], metavar="NAME=VALUE",
                    help="library tuning knob (dlm_set_option) applied before the run; may be repeated")
    ap.add_argument("--ab", default=None, metavar="NAME=V1,V2[,...]",
                    help="A/B inside one process (boxes of the pool differ by a few percent, runs on one box repeat within "
                         "0.2 %%): after the clock ramp, alternate the values of a dlm_set_option knob (or of the rollout driver's "
                         "'expect_ratio', its row-count guess, or 'predict_finish'), --steps steps each, three rounds; prints one JSON line per "
                         "measurement and returns")
    ap.add_argument("--dump-steps", default=None, metavar="FILE",
                    help="write one line per sampled step: block, rows masked before / after, active sequences, "
                         "attention / LM-head / commit call in us")
    ap.add_argument("--kernel", default=None, choices=["lmhead", "attn_fullseq", "fullpass", "kv_refresh", "peaks", "attn", "gemm_ref"],
                    help="time ONE library call on random inputs instead of the rollout (record only, for profiles): "
                         "lmhead = dlm_lmhead_confidence at --rows rows on the config's W shape; attn = dlm_block_attn at the "
                         "config's rollout shape (last block); attn_fullseq = dlm_block_attn (and, with --backward, "
                         "dlm_block_attn_bwd) on 64 x 4096 tokens, 32/8 heads, d = 128; fullpass = one full-sequence "
                         "block-diffusion pass of workload c5b (attention, row compaction, LM head on the masked rows, one "
                         "commit per block of 4), each part timed; kv_refresh = dlm_kv_refresh on the cache images of c2, "
                         "c3, c4 and c5; peaks = device copy, one-pass read and register-only MFMA loop; gemm_ref = torch.matmul (the vendor "
                         "GEMM) on the LM head's operand shapes, for context")
    ap.add_argument("--shape", default=None, metavar="B,Hq,Hkv,Lq,Lk", help="--kernel attn: this shape (d = 128, full mask) instead of the config's")
    ap.add_argument("--rows", type=int, default=8192, help="--kernel lmhead: number of hidden rows M")
    ap.add_argument("--lmhead-variant", default="-1", help="--kernel lmhead: comma-separated entries of the shape table (-1 = planner)")
    ap.add_argument("--zeros", action="store_true", help="--kernel lmhead: all-zero operands (no data-dependent power)")
    ap.add_argument("--mask", default="block_causal", choices=["full", "block_causal"], help="--kernel attn_fullseq")
    ap.add_argument("--batch", type=int, default=64, help="--kernel attn_fullseq: sequences")
    ap.add_argument("--backward", action="store_true", help="--kernel attn_fullseq: also time the backward pass")
    ap.add_argument("--reps", type=int, default=3, help="--kernel: timed calls per measurement")
    return ap.parse_args()


# ---------------------------------------------------------------------------------------------------------- #
# achievable peaks (libdlm_peaks: plain copy, one-pass read, register-only MFMA loop)
# ---------------------------------------------------------------------------------------------------------- #
def measure_peaks(torch, reps: int = 20) -> dict:
    from paper_2604_04215_amd.build import PEAKS_LIB
    if not os.path.exists(PEAKS_LIB):
        raise RuntimeError(f"{PEAKS_LIB} not found: build it with `python -m paper_2604_04215_amd.build`")
    L = C.CDLL(PEAKS_LIB)
    L.dlm_peak_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_void_p]
    L.dlm_peak_read.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_void_p, C.c_void_p]
    L.dlm_peak_mfma.argtypes = [C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
    dev = "cuda:0"
    nbytes = 1 << 30
    src = torch.randint(0, 255, (nbytes,), dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    sink = torch.zeros(nbytes // 16384 + 16, dtype=torch.int32, device=dev)
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)

    def timed(fn):
        for _ in range(3):
            assert fn() == 0
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e-3

    out = {}
    t = timed(lambda: L.dlm_peak_copy(src.data_ptr(), dst.data_ptr(), nbytes, 0, st))
    out["copy_gbs"] = round(2 * nbytes / t / 1e9, 1)               # read + write
    t = timed(lambda: L.dlm_peak_read(src.data_ptr(), nbytes, 0, sink.data_ptr(), st))
    out["read_gbs"] = round(nbytes / t / 1e9, 1)
    t = timed(lambda: L.dlm_peak_read(src.data_ptr(), nbytes, 1, sink.data_ptr(), st))
    out["read_nt_gbs"] = round(nbytes / t / 1e9, 1)
    n_wg, iters = 256 * 8, 4096
    fs = torch.zeros(n_wg * 4, dtype=torch.float32, device=dev)
    t = timed(lambda: L.dlm_peak_mfma(n_wg, iters, None, fs.data_ptr(), st))
    out["mfma_bf16_tflops"] = round(n_wg * 4 * iters * 8 * 32768 / t / 1e12, 1)
    ops = torch.randn(16 * 64 * 8, device=dev).bfloat16()          # N(0,1) operand fragments
    t = timed(lambda: L.dlm_peak_mfma(n_wg, iters, ops.data_ptr(), fs.data_ptr(), st))
    out["mfma_bf16_tflops_normal_data"] = round(n_wg * 4 * iters * 8 * 32768 / t / 1e12, 1)
    # do MFMA and vector-ALU work overlap on a SIMD: across wavefronts (mode 2) / inside one wavefront's stream (mode 3)?
    L.dlm_peak_overlap.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
    ov = {}
    for mode, key in ((0, "all_mfma"), (1, "all_valu"), (2, "mfma_waves_beside_valu_waves"), (3, "both_in_each_wave")):
        ov[key] = round(timed(lambda: L.dlm_peak_overlap(mode, 256, 20000, fs.data_ptr(), st)) * 1e3, 3)
    ov["note"] = ("ms for 20000 iterations, 8 wavefronts per CU; side by side across wavefronts would give max(all_mfma, all_valu) / 2 "
                  "for the third figure, mutual exclusion their sum / 2")
    out["mfma_valu_overlap_ms"] = ov
    out["what"] = ("1 GiB device copy (read + write), 1 GiB one-pass read with ordinary / non-temporal loads, "
                   "register-only 32x32x16 bf16 MFMA loop on 2048 workgroups of 4 wavefronts with small constant operands and "
                   "with N(0,1) operands (the power limit lowers the clock on realistic data)")
    return out


def micro(args):
    """One kernel on random inputs (normal bf16 values, the rollout's W scale): a JSON line per measurement."""
    import torch
    from paper_2604_04215_amd import binding as dlm
    from paper_2604_04215_amd import synth
    dlm.lib()
    dev = "cuda:0"
    torch.manual_seed(0)

    blocker = torch.randn(8192, 8192, device=dev).bfloat16() if args.kernel in ("attn", "kv_refresh") else None

    def timed(fn, reps):
        # untimed calls first, about 80 ms of them: the clock of an idle GPU takes tens of milliseconds of work to come up
        # (the first shape measured in a process otherwise reads 10 - 20 % slow)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn()
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        for _ in range(min(400, int(80.0 / max(e0.elapsed_time(e1), 0.01)))):
            fn()
        torch.cuda.synchronize()
        if blocker is not None:
            # calls of a few tens of microseconds: a few milliseconds of unrelated work go first, so that the host has
            # queued every timed call before the first one starts and the events measure GPU time, not the Python loop
            for _ in range(6):
                torch.mm(blocker, blocker)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    if args.kernel == "peaks":
        print(json.dumps({"kernel": "peaks", **measure_peaks(torch, max(args.reps, 10))}), flush=True)
        return
    if args.kernel == "gemm_ref":
        # context only: the vendor GEMM (torch.matmul -> hipBLASLt) on the LM head's operand shapes, N(0,1)-scaled data and
        # zeros: what a plain [M, Dh] x [Dh, V] product (logits written to HBM, no softmax) sustains on this machine
        cfg = synth.CONFIGS[args.config]
        V, Dh = cfg.V, cfg.Dh
        for M in (512, 1024, 8192):
            for data in ("normal", "zeros"):
                if data == "normal":
                    w = (torch.randn((V, Dh), device=dev) * Dh ** -0.25).bfloat16()
                    h = torch.randn((M, Dh), device=dev).bfloat16()
                else:
                    w = torch.zeros((V, Dh), device=dev, dtype=torch.bfloat16)
                    h = torch.zeros((M, Dh), device=dev, dtype=torch.bfloat16)
                out = torch.empty((M, V), device=dev, dtype=torch.bfloat16)
                ms = timed(lambda: torch.matmul(h, w.t(), out=out), max(args.reps, 5))
                print(json.dumps({"kernel": "torch.matmul (vendor GEMM, reference only)", "M": M, "V": V, "Dh": Dh, "data": data,
                                  "us": round(ms * 1e3, 1), "tflops": round(2.0 * M * V * Dh / ms / 1e9, 1),
                                  "frac_mfma_peak": round(2.0 * M * V * Dh / ms / 1e9 / MFMA_PEAK_TFLOPS, 3)}), flush=True)
                del w, h, out
        return
    if args.kernel == "kv_refresh":
        # the block-boundary cache refresh of every rollout workload: the prefix (and, dual cache, suffix) image
        for name, B, Hkv, L, rows in (("c2 prefix at the last block", 8, 32, 768, 736), ("c3 prefix + suffix", 16, 32, 1536, 1504),
                                      ("c4-sized cache", 32, 4, 1024, 992), ("c5 cache", 64, 8, 4096, 4092)):
            src_k = torch.randn((B, Hkv, L, 128), device=dev).bfloat16()
            src_v = torch.randn((B, Hkv, L, 128), device=dev).bfloat16()
            ck, cv = torch.empty_like(src_k), torch.empty_like(src_v)
            ms = timed(lambda: dlm.kv_refresh(src_k[:, :, :rows], src_v[:, :, :rows], ck, cv, 0), max(args.reps, 10))
            moved = 2 * 2 * B * Hkv * rows * 128 * 2          # K and V, read + write
            print(json.dumps({"kernel": "dlm_kv_refresh", "workload": name, "B": B, "Hkv": Hkv, "rows": rows, "d": 128,
                              "bytes_read_plus_written": moved, "us": round(ms * 1e3, 1),
                              "gbs": round(moved / ms / 1e6, 1), "frac_hbm_peak": round(moved / ms / 1e6 / HBM_PEAK_GBS, 3)}),
                  flush=True)
            del src_k, src_v, ck, cv
        return
    if args.kernel == "attn":
        cfg = synth.CONFIGS[args.config]
        blk = cfg.n_blocks - 1
        if args.shape:       # B,Hq,Hkv,Lq,Lk: a full-mask block of Lq rows against Lk - Lq cached keys plus itself
            B_, Hq_, Hkv_, Lq_, Lk_ = (int(x) for x in args.shape.split(","))
            cfg = cfg.replace(name="shape " + args.shape, B=B_, Hq=Hq_, Hkv=Hkv_, d=128, Lb=Lq_, prompt=Lk_ - Lq_, gen=Lq_,
                              dual_cache=False, mask_mode="full", bs=0)
            blk = 0
        P = cfg.prompt + blk * cfg.Lb
        S = cfg.L - P - cfg.Lb if cfg.dual_cache else 0
        mk = lambda *shape: torch.randn(shape, device=dev).bfloat16()
        ck, cv = mk(cfg.B, cfg.Hkv, cfg.L, cfg.d), mk(cfg.B, cfg.Hkv, cfg.L, cfg.d)
        q, kb, vb = mk(cfg.B, cfg.Lb, cfg.Hq, cfg.d), mk(cfg.B, cfg.Hkv, cfg.Lb, cfg.d), mk(cfg.B, cfg.Hkv, cfg.Lb, cfg.d)
        out = torch.empty_like(q)
        mode = dlm.MASK_FULL if cfg.mask_mode == "full" else dlm.MASK_BLOCK_CAUSAL
        suffix = (ck[:, :, P + cfg.Lb:], cv[:, :, P + cfg.Lb:], P + cfg.Lb) if S > 0 else None
        ws_bytes = dlm.block_attn_workspace_bytes(q, prefix=(ck[:, :, :P], cv[:, :, :P], 0), block=(kb, vb, P), suffix=suffix,
                                                  mask_mode=mode, block_size=cfg.bs, q_pos0=P)
        ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
        ms = timed(lambda: dlm.block_attn(q, out, prefix=(ck[:, :, :P], cv[:, :, :P], 0), block=(kb, vb, P), suffix=suffix,
                                          mask_mode=mode, block_size=cfg.bs, q_pos0=P, workspace=ws), max(args.reps, 20))
        Lk = P + cfg.Lb + S
        nbytes, flop = attn_cost(cfg, cfg.B, Lk)
        print(json.dumps({"kernel": "dlm_block_attn", "workload": f"{cfg.name} rollout step, last block", "B": cfg.B,
                          "heads": [cfg.Hq, cfg.Hkv], "Lq": cfg.Lb, "Lk": Lk, "workspace_bytes": ws_bytes,
                          "key_splits": ws_bytes // (cfg.B * cfg.Hq * cfg.Lb * (cfg.d + 2) * 4) if ws_bytes else 1,
                          "options": args.set_option,
                          "us": round(ms * 1e3, 1), "gbs": round(nbytes / ms / 1e6, 1), "tflops": round(flop / ms / 1e9, 1),
                          "frac_hbm_peak": round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 3),
                          "frac_mfma_peak": round(flop / ms / 1e9 / MFMA_PEAK_TFLOPS, 3)}), flush=True)
        return
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
            nbytes, flop = lmhead_cost(cfg, M)
            print(json.dumps({"kernel": "dlm_lmhead_confidence", "M": M, "V": V, "Dh": Dh, "variant": variant,
                              "data": "zeros" if args.zeros else "normal", "us": round(ms * 1e3, 1),
                              "tflops": round(flop / ms / 1e9, 1), "frac_mfma_peak": round(flop / ms / 1e9 / MFMA_PEAK_TFLOPS, 3),
                              "gbs": round(nbytes / ms / 1e6, 1), "frac_hbm_peak": round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 3),
                              "bound": "mfma" if flop / nbytes >= RIDGE else "hbm"}), flush=True)
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
                rec["frac_mfma_peak"] = round(flop / ms / 1e9 / MFMA_PEAK_TFLOPS, 3)
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
                      "ms": round(ms, 3), "tflops": round(4.0 * B * Hq * d * pairs / ms / 1e9, 1),
                      "frac_mfma_peak": round(4.0 * B * Hq * d * pairs / ms / 1e9 / MFMA_PEAK_TFLOPS, 3)}), flush=True)
    if args.backward:
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        ws = torch.empty(dlm.block_attn_bwd_workspace_bytes(B * L, Hq), dtype=torch.uint8, device=dev)
        ms = timed(lambda: dlm.block_attn_bwd(q, out, do, lse, dq, block=(k, v, 0), d_block=(dk, dv), mask_mode=mode,
                                              block_size=bs, workspace=ws), args.reps)
        print(json.dumps({"kernel": "dlm_block_attn_bwd", "mask": args.mask, "B": B, "L": L, "heads": [Hq, Hkv], "d": d,
                          "ms": round(ms, 3), "tflops": round(10.0 * B * Hq * d * pairs / ms / 1e9, 1)}), flush=True)


# ---------------------------------------------------------------------------------------------------------- #
# algorithmic bytes / FLOP of one call
# ---------------------------------------------------------------------------------------------------------- #
def attn_cost(cfg, active_seqs, Lk):
    """K and V once per KV head, Q read, O written; 4 * d FLOP per visible (query, key) pair and query head.  Every
    rollout workload's query block sees all Lk keys (the block-causal one denoises the last block)."""
    nbytes = active_seqs * (2 * cfg.Hkv * Lk * cfg.d * 2 + 2 * cfg.Lb * cfg.Hq * cfg.d * 2)
    flop = 4.0 * active_seqs * cfg.Hq * cfg.d * cfg.Lb * Lk
    return nbytes, flop


def lmhead_cost(cfg, rows):
    """W_vocab once, the gathered hidden rows, 8 bytes of outputs per row; 2 * Dh * V FLOP per row."""
    return cfg.V * cfg.Dh * 2 + rows * cfg.Dh * 2 + rows * 8, 2.0 * rows * cfg.Dh * cfg.V


def commit_cost(cfg, copied_seqs):
    """Per position: confidence, token, mask in and out, commit flag, next-row list (18 B); per copied sequence the
    block's K and V read and written."""
    return cfg.B * cfg.Lb * 18 + copied_seqs * 2 * 2 * cfg.Hkv * cfg.Lb * cfg.d * 2, 0.0


def roof_record(name, us_list, bytes_list, flop_list, measured):
    """Aggregate of one call over the sampled steps: total algorithmic work / total measured time, against the roof
    that binds at the aggregate arithmetic intensity (nominal peaks), and against the measured peaks."""
    n = len(us_list)
    if n == 0:
        return None
    tot_s = sum(us_list) * 1e-6
    tot_b, tot_f = float(sum(bytes_list)), float(sum(flop_list))
    gbs = tot_b / tot_s / 1e9
    tfl = tot_f / tot_s / 1e12
    ai = tot_f / tot_b if tot_b else 0.0
    bound = "mfma" if ai >= RIDGE else "hbm"
    rec = {"call": name, "calls": n, "avg_us": round(sum(us_list) / n, 2), "median_us": round(sorted(us_list)[n // 2], 2),
           "bytes_per_call": int(tot_b / n), "flop_per_call": int(tot_f / n), "intensity_flop_per_byte": round(ai, 1),
           "bound": bound, "gbs": round(gbs, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
           "tflops": round(tfl, 1), "frac_mfma_peak": round(tfl / MFMA_PEAK_TFLOPS, 4),
           # the most the other roof's fraction could be at this intensity
           "ceiling_frac_mfma_peak": round(min(1.0, ai / RIDGE), 4), "ceiling_frac_hbm_peak": round(min(1.0, RIDGE / ai) if ai else 1.0, 4),
           "frac": round((tfl / MFMA_PEAK_TFLOPS) if bound == "mfma" else (gbs / HBM_PEAK_GBS), 4)}
    if measured:
        ref_bw = measured["copy_gbs"] if name in ("dlm_unmask_commit", "dlm_kv_refresh") else measured["read_nt_gbs"]
        rec["frac_of_measured_hbm"] = round(gbs / ref_bw, 4)
        rec["frac_of_measured_mfma"] = round(tfl / measured["mfma_bf16_tflops_normal_data"], 4)   # the loop on N(0,1) operands
    return rec


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
    cfg = synth.CONFIGS[args.config].replace(w_dist=args.w_dist)
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

    # ---- clock ramp + warm-up, then the timed region (nothing but the steps' own launches inside) ----
    ramp_done = 0
    if args.ramp_steps > 0:
        t_ramp = time.perf_counter()
        while True:
            runner.run(args.ramp_steps)
            ramp_done += args.ramp_steps
            torch.cuda.synchronize()
            if time.perf_counter() - t_ramp >= args.ramp_seconds or ramp_done >= 200 * args.ramp_steps:
                break
        # ... and ends where a rollout ends, so that the warm-up and the timed region always begin at the same place of the
        # rollout whatever the length of the ramp was (a short timed region covers a fraction of a rollout, whose early
        # steps commit many tokens and its late ones few)
        while runner.in_block or runner.block != cfg.n_blocks - 1:
            runner.run(1)
            ramp_done += 1
    if args.warmup > 0:
        runner.run(args.warmup)
    torch.cuda.synchronize()
    if args.ab:
        name, _, vals = args.ab.partition("=")
        for rnd in range(3):
            for v in vals.split(","):
                if name == "expect_ratio":
                    g.expect_ratio = float(v)
                elif name == "predict_finish":
                    g.predict_finish = bool(int(v))
                else:
                    dlm.set_option(name, int(v))
                runner.run(max(50, args.steps // 10))       # the new setting's own warm-up
                torch.cuda.synchronize()
                ta = time.perf_counter()
                runner.run(args.steps)
                torch.cuda.synchronize()
                tb = time.perf_counter()
                print(json.dumps({"ab": name, "value": v, "round": rnd, "workload": cfg.name, "steps": args.steps,
                                  "us_per_step": round((tb - ta) / args.steps * 1e6, 2)}), flush=True)
        return
    c0, e0 = runner.committed, runner.empty
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    res = runner.run(args.steps)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    elapsed = t1 - t0
    committed = runner.committed - c0
    empty = runner.empty - e0
    assert res["steps"] == args.steps

    # ---- achievable peaks on this machine (own kernels, a few ms each) ------------------------------------
    measured = None
    if not args.no_peaks:
        measured = measure_peaks(torch)

    # ---- per-call sample pass: a fixed number of steps, every library call between two events --------
    kernels, roof, sample_info = {}, None, None
    if args.sample_steps > 0:
        ev = {n: [] for n in ("block_attn", "lmhead_confidence", "unmask_commit", "kv_refresh")}
        cap = args.sample_steps + 8 * cfg.n_blocks * (args.sample_steps // max(1, rollout_steps) + 2) + 64
        rem_hist = torch.zeros((cap, cfg.B), dtype=torch.int32, device=dev)   # per-sequence still-masked counts after each step
        n_commit_calls = [0]

        def on_call(name, fn, a, sp, meta):
            """stands in for one library call of a step: the same call between two events on the launch stream"""
            a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            st = torch.cuda.current_stream()
            a0.record(st)
            rc = fn(*a, sp) if name == "kv_refresh" else fn(C.byref(a), sp)
            a1.record(st)
            if name == "block_attn":
                meta = dict(first=meta["first"], Lk=a.prefix.len + a.block.len + a.suffix.len, prev=n_commit_calls[0] - 1)
            elif name == "unmask_commit":
                i = n_commit_calls[0]
                n_commit_calls[0] += 1
                rem_hist[i].copy_(meta["remaining"])       # after the bracketed call: the counts of this step
                meta = dict(idx=i, first=meta["first"])
            ev[name].append((a0, a1, meta))
            return rc

        g.on_call = on_call
        log0 = len(runner.log)
        try:
            runner.run(args.sample_steps)
            torch.cuda.synchronize()
        finally:
            g.on_call = None
        log = runner.log[log0:]
        # the runner polls every step it queued except possibly the last one or two of an unfinished block
        n_steps = min(len(log), len(ev["lmhead_confidence"]))
        hist = rem_hist[:n_commit_calls[0]].cpu().numpy()
        us = lambda e: e[0].elapsed_time(e[1]) * 1e3
        at = dict(us=[], b=[], f=[])
        lm = dict(us=[], b=[], f=[], rows=[])
        cm = dict(us=[], b=[], f=[])
        lines = []
        for i in range(n_steps):
            blk, before, after = log[i]
            ea, el, ec = ev["block_attn"][i], ev["lmhead_confidence"][i], ev["unmask_commit"][i]
            am, cmeta = ea[2], ec[2]
            active = cfg.B if (am["first"] or am["prev"] < 0) else int((hist[am["prev"]] > 0).sum())
            if before <= 0:
                continue                     # a queued step that found nothing masked moves no data
            b_, f_ = attn_cost(cfg, active, am["Lk"])
            at["us"].append(us(ea)); at["b"].append(b_); at["f"].append(f_)
            b_, f_ = lmhead_cost(cfg, before)
            lm["us"].append(us(el)); lm["b"].append(b_); lm["f"].append(f_); lm["rows"].append(before)
            copied = int((hist[cmeta["idx"]] == 0).sum()) - (cfg.B - active) if cmeta["first"] else active
            b_, f_ = commit_cost(cfg, max(copied, 0))
            cm["us"].append(us(ec)); cm["b"].append(b_); cm["f"].append(f_)
            lines.append(f"{blk} {before} {after} {active} {us(ea):.1f} {us(el):.1f} {us(ec):.1f}")
        if args.dump_steps:
            with open(args.dump_steps, "w") as f:
                f.write("\n".join(lines) + "\n")
        rf = ev["kv_refresh"]
        kernels = {"dlm_block_attn": roof_record("dlm_block_attn", at["us"], at["b"], at["f"], measured),
                   "dlm_lmhead_confidence": roof_record("dlm_lmhead_confidence", lm["us"], lm["b"], lm["f"], measured),
                   "dlm_unmask_commit": roof_record("dlm_unmask_commit", cm["us"], cm["b"], cm["f"], measured),
                   "dlm_kv_refresh": roof_record("dlm_kv_refresh", [us(e) for e in rf], [e[2]["bytes"] for e in rf],
                                                 [0.0] * len(rf), measured)}
        if kernels["dlm_lmhead_confidence"]:
            kernels["dlm_lmhead_confidence"]["mean_rows"] = round(sum(lm["rows"]) / len(lm["rows"]), 1)
        if kernels["dlm_unmask_commit"]:
            kernels["dlm_unmask_commit"]["note"] = "selection + commit + row compaction + block K/V write-back in one launch: launch-latency-bound, bytes are the ones it touches"
        sample_info = {"steps": len(lm["us"]), "events": "torch.cuda.Event pairs on the launch stream around every library call, after the timed region"}
        # the call that takes most of a step is the one the roofline object describes
        dom = max((k for k in kernels.values() if k and k["call"] != "dlm_kv_refresh"), key=lambda k: k["avg_us"] * k["calls"])
        peak, unit, ach = (MFMA_PEAK_TFLOPS, "TFLOP/s", dom["tflops"]) if dom["bound"] == "mfma" else (HBM_PEAK_GBS, "GB/s", dom["gbs"])
        other = ({"bound": "hbm", "achieved": dom["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": dom["frac_hbm_peak"],
                  "ceiling_frac": dom["ceiling_frac_hbm_peak"]} if dom["bound"] == "mfma" else
                 {"bound": "mfma", "achieved": dom["tflops"], "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": dom["frac_mfma_peak"],
                  "ceiling_frac": dom["ceiling_frac_mfma_peak"]})
        kern_names = {"dlm_lmhead_confidence": "lmhead_kernel (M <= 256) or lmhead_pair_kernel (above) + lmhead_reduce_kernel (one dlm_lmhead_confidence call)",
                      "dlm_block_attn": "attn_kernel (one dlm_block_attn call)",
                      "dlm_unmask_commit": "commit_fused_kernel (one dlm_unmask_commit call)"}
        roof = dict(bound=dom["bound"], achieved=ach, peak=peak, unit=unit, frac=round(ach / peak, 4),
                    traffic=int(LMHEAD_C2_TRAFFIC_BYTES) if (args.config == "c2" and args.w_dist == "var" and dom["call"] == "dlm_lmhead_confidence") else None,
                    kernel=kern_names[dom["call"]], call=dom["call"], avg_us=dom["avg_us"], median_us=dom["median_us"],
                    launches=dom["calls"], bytes_per_launch=dom["bytes_per_call"], flops_per_launch=dom["flop_per_call"],
                    intensity_flop_per_byte=dom["intensity_flop_per_byte"], other_roof=other)
        if dom["call"] == "dlm_lmhead_confidence":
            roof["mean_rows"] = kernels["dlm_lmhead_confidence"]["mean_rows"]
        if measured:
            roof["frac_of_measured_peak"] = dom["frac_of_measured_mfma"] if dom["bound"] == "mfma" else dom["frac_of_measured_hbm"]

    # ---- CPU oracle on a bounded sample of the same workload ----------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        tc0 = time.perf_counter()
        n_tok = n_steps_cpu = n_seq = 0
        want = min(args.oracle_seqs, cfg.B) if args.oracle_seqs > 0 else cfg.B
        for b in range(want):                        # whole sequences of block 0, one at a time
            o = oracle.OracleRollout(cfg, synth, seqs=[b], w=w_host)
            o.begin_block(0)
            while o.mask.any():
                r = o.step()
                n_tok += int(r["n_commit"].sum())
                n_steps_cpu += 1
            n_seq += 1
            if args.oracle_seqs <= 0 and time.perf_counter() - tc0 > 12.0:
                break
        tc = time.perf_counter() - tc0
        full_s = tc * cfg.B / n_seq * cfg.n_blocks
        cpu = dict(value=round(n_tok / tc, 3), unit="committed tokens/s", cores=oracle.num_threads(), kind="oracle",
                   sample=f"sequences 0..{n_seq - 1} of the batch, one at a time, block 0 (prefix {cfg.prompt} + block "
                          f"{cfg.Lb}) to completion: {n_steps_cpu} denoising steps, {n_tok} tokens committed in {tc:.1f} s",
                   measured_s=round(tc, 2),
                   extrapolated_whole_rollout_s=round(full_s, 1),
                   extrapolation=f"linear: measured time x (B={cfg.B} / {n_seq} sequences) x {cfg.n_blocks} blocks; later blocks "
                                 "have longer prefixes, so this is a lower estimate")

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
        "config": {"workload": WORKLOADS[args.config] + ("" if args.w_dist == "var" else " [W_vocab std reading]"),
                   "committed_tokens": committed, "tokens_per_step": round(committed / args.steps, 3),
                   "steps_per_rollout": rollout_steps, "steps_per_block": steps_per_block,
                   "empty_steps_in_timed_region": empty, "ramp_steps": ramp_done,
                   "loop": "sync" if args.sync_loop else "one-step-late poll", "setup_s": round(setup_s, 1)},
        "roofline": roof,
        "kernels": kernels,
        "kernel_sample": sample_info,
        "peaks": {"nominal": {"hbm_gbs": HBM_PEAK_GBS, "mfma_bf16_tflops": MFMA_PEAK_TFLOPS}, "measured": measured},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
