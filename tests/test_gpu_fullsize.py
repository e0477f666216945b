"""The five benchmark workloads at their full sizes, in the launch configuration the benchmark uses
(GpuRollout.step); the oracle checks sampled outputs one by one, properties cover the rest (GPU)."""
import numpy as np
import pytest
import torch

import oracle
from oracle import KV
from oracle.denoise import apply_commit, select_commit
from paper_2604_04215_amd import binding as dlm
from paper_2604_04215_amd import synth
from paper_2604_04215_amd.rollout import GpuRollout
from gpu_util import DEV, attn_err_report, bf16_dev, bf16_host, dev, fmt_err

pytestmark = pytest.mark.gpu

ATTN_TOL, CONF_TOL, NEAR = 2e-2, 1e-3, 1e-3


def check_attn_rows(got_O, ref_rows_O, rows):
    got = synth.bf16_bits_to_f64(np.stack([got_O[b, i, h] for b, h, i in rows]))
    rms = np.sqrt((ref_rows_O ** 2).mean(axis=-1, keepdims=True))
    err = (np.abs(got - ref_rows_O) / np.maximum(np.abs(ref_rows_O), rms)).max()
    assert err <= ATTN_TOL, f"attention rel err {err}"


def check_lm_rows(conf_g, tok_g, ref):
    assert np.abs(conf_g.astype(np.float64) - ref["conf"]).max() <= CONF_TOL
    clear = (ref["zmax"] - ref["z2nd"]) >= NEAR
    assert np.array_equal(tok_g[clear], ref["tok"][clear])


def run_rollout_step(name, block, n_attn_rows=24, n_lm_rows=6):
    cfg = synth.CONFIGS[name]
    rng = np.random.default_rng(cfg.seed)
    w = synth.w_vocab(cfg)
    g = GpuRollout(cfg, bf16_dev(w), DEV)
    k, v = synth.cache_kv(cfg, block)
    g.cache_k.copy_(bf16_dev(k))
    g.cache_v.copy_(bf16_dev(v))
    x0 = synth.initial_tokens(cfg, cfg.L)
    g.x.copy_(dev(x0))
    g.begin_block(block)
    P, Lb, S = g.P, cfg.Lb, g.S
    q = synth.step_q(cfg, block, 0)
    kb, vb = synth.step_kv(cfg, block, 0)
    hid = synth.step_hidden(cfg, block, 0)
    g.step(bf16_dev(q), bf16_dev(kb), bf16_dev(vb), bf16_dev(hid))
    torch.cuda.synchronize()

    # attention: sampled (b, h, i) rows against the oracle
    segs = [KV(k[:, :, :P], v[:, :, :P], 0), KV(kb, vb, P)]
    if S > 0:
        segs.append(KV(k[:, :, P + Lb:P + Lb + S], v[:, :, P + Lb:P + Lb + S], P + Lb))
    rows = np.stack([rng.integers(0, cfg.B, n_attn_rows), rng.integers(0, cfg.Hq, n_attn_rows),
                     rng.integers(0, Lb, n_attn_rows)], axis=1).astype(np.int32)
    rows[0] = (cfg.B - 1, cfg.Hq - 1, Lb - 1)
    ref_O, ref_lse = oracle.attention(q, segs, mask_mode=cfg.mask_mode, bs=cfg.bs, q_pos0=P, rows=rows)
    check_attn_rows(bf16_host(g.O), ref_O, rows)
    lse_g = g.lse_attn.cpu().numpy()
    assert np.abs(np.array([lse_g[b, h, i] for b, h, i in rows]) - ref_lse).max() <= 2e-3

    # LM head: every row was masked; sampled rows against the oracle
    conf_g, tok_g = g.conf.cpu().numpy().ravel(), g.tok.cpu().numpy().ravel()
    sample = np.unique(np.concatenate([[0, cfg.B * Lb - 1], rng.integers(0, cfg.B * Lb, n_lm_rows)])).astype(np.int32)
    ref = oracle.lmhead(hid.reshape(cfg.B * Lb, cfg.Dh), w, row_idx=sample, forbid_token=cfg.forbid_token)
    check_lm_rows(conf_g[sample], tok_g[sample], ref)
    assert np.all((tok_g >= 0) & (tok_g < cfg.V - 1)) and np.all((conf_g > 0) & (conf_g <= 1 + 1e-6))
    zmax, lse = g.zmax.cpu().numpy(), g.lse.cpu().numpy()
    assert np.allclose(conf_g, np.exp(zmax - lse), atol=1e-5)

    # selection and commit: the oracle's rule on the confidences the GPU produced is exact
    mask0 = np.ones((cfg.B, Lb), np.uint8)
    commit, n_commit, remaining = select_commit(conf_g.reshape(cfg.B, Lb).astype(np.float64), mask0, rule=cfg.rule,
                                                tau=float(np.float32(cfg.tau)), k=cfg.k)
    x_ref, m_ref = x0.copy(), mask0.copy()
    apply_commit(x_ref, P, m_ref, tok_g.reshape(cfg.B, Lb), commit)
    assert np.array_equal(g.commit_now.cpu().numpy(), commit)
    assert np.array_equal(g.x.cpu().numpy(), x_ref) and np.array_equal(g.mask.cpu().numpy(), m_ref)
    assert np.array_equal(g.n_commit.cpu().numpy(), n_commit) and np.array_equal(g.remaining.cpu().numpy(), remaining)
    assert np.all(n_commit >= 1)
    flat = np.flatnonzero(m_ref.ravel())
    assert int(g.m_dev.item()) == len(flat) and np.array_equal(g.row_idx.cpu().numpy()[:len(flat)], flat)
    # cache untouched unless a sequence finished in this very step
    done = (remaining == 0) & (n_commit > 0)
    ck = bf16_host(g.cache_k)
    for b in range(cfg.B):
        want = kb[b] if done[b] else k[b, :, P:P + Lb]
        assert np.array_equal(ck[b, :, P:P + Lb], want)
    return g


def test_c2_llada8b_step_last_block():
    run_rollout_step("c2", block=7)


def test_c3_dual_cache_step():
    run_rollout_step("c3", block=5)


def test_c4_dream7b_gqa_topk_step():
    g = run_rollout_step("c4", block=7)
    assert np.all(g.n_commit.cpu().numpy() == 4)


def test_c5a_block_causal_rollout_step():
    run_rollout_step("c5a", block=0, n_attn_rows=16)


def test_c5b_full_sequence_block_causal_pass():
    """64 x 4096 tokens, block size 4, Bernoulli(0.5) masking: attention over the whole sequence,
    LM head on the ~131k masked rows, one threshold commit per block of 4."""
    cfg = synth.FULLPASS["c5b"]
    rng = np.random.default_rng(cfg.seed)
    B, L = cfg.B, cfg.L
    w = synth.w_vocab(cfg)
    q, k, v = synth.fullpass_qkv(cfg)
    hid = synth.fullpass_hidden(cfg)
    mask0 = synth.fullpass_mask(cfg)
    x0 = synth.initial_tokens(cfg, L)
    print("inputs drawn", flush=True)
    w_d, q_d, k_d, v_d = bf16_dev(w), bf16_dev(q), bf16_dev(k), bf16_dev(v)
    hid_d = bf16_dev(hid).view(B * L, cfg.Dh)
    out = torch.empty((B, L, cfg.Hq, cfg.d), dtype=torch.bfloat16, device=DEV)
    dlm.block_attn(q_d, out, block=(k_d, v_d, 0), mask_mode=dlm.MASK_BLOCK_CAUSAL, block_size=cfg.bs, q_pos0=0)
    mask = dev(mask0)
    row_idx = torch.zeros(B * L, dtype=torch.int32, device=DEV)
    m_dev = torch.zeros(1, dtype=torch.int32, device=DEV)
    dlm.mask_compact(mask, row_idx, m_dev)
    conf = torch.zeros((B, L), dtype=torch.float32, device=DEV)
    tok = torch.zeros((B, L), dtype=torch.int32, device=DEV)
    torch.cuda.synchronize()
    M = int(m_dev.item())
    assert M == int(mask0.sum()) and abs(M / (B * L) - 0.5) < 0.01
    ws = torch.empty(dlm.lmhead_workspace_bytes(M, cfg.V), dtype=torch.uint8, device=DEV)
    dlm.lmhead_confidence(hid_d, w_d, conf, tok, M=M, row_idx=row_idx, forbid_token=cfg.forbid_token,
                          out_scatter=True, workspace=ws)
    x = dev(x0)
    n_commit = torch.zeros(B, dtype=torch.int32, device=DEV)
    remaining = torch.zeros(B, dtype=torch.int32, device=DEV)
    commit_now = torch.zeros((B, L), dtype=torch.uint8, device=DEV)
    dlm.unmask_commit(conf, tok, x, mask, n_commit, remaining, x_pos0=0, group_len=cfg.bs,
                      rule=dlm.RULE_THRESHOLD, threshold=cfg.tau, commit_now=commit_now)
    torch.cuda.synchronize()
    print("gpu pass done", flush=True)

    # attention rows (early, middle, last blocks) against the oracle
    n = 20
    rows = np.stack([rng.integers(0, B, n), rng.integers(0, cfg.Hq, n), rng.integers(0, L, n)], axis=1).astype(np.int32)
    rows[0], rows[1], rows[2] = (0, 0, 0), (B - 1, cfg.Hq - 1, L - 1), (3, 5, 4)
    ref_O, _ = oracle.attention(q, [KV(k, v, 0)], mask_mode="block_causal", bs=cfg.bs, q_pos0=0, rows=rows)
    check_attn_rows(bf16_host(out), ref_O, rows)
    # LM head: sampled masked rows
    flat_masked = np.flatnonzero(mask0.ravel())
    sample = np.unique(np.concatenate([[flat_masked[0], flat_masked[-1]], rng.choice(flat_masked, 6)])).astype(np.int32)
    ref = oracle.lmhead(hid.reshape(B * L, cfg.Dh), w, row_idx=sample, forbid_token=cfg.forbid_token)
    conf_g, tok_g = conf.cpu().numpy(), tok.cpu().numpy()
    check_lm_rows(conf_g.ravel()[sample], tok_g.ravel()[sample], ref)
    # selection: exact on three whole sequences given the GPU's confidences; group properties on all
    commit_g = commit_now.cpu().numpy()
    for b in (0, 31, 63):
        commit, nc, rem = select_commit(conf_g[b:b + 1].astype(np.float64), mask0[b:b + 1], rule="threshold",
                                        tau=float(np.float32(cfg.tau)), group_len=cfg.bs)
        assert np.array_equal(commit_g[b:b + 1], commit)
        assert int(n_commit[b].item()) == nc[0] and int(remaining[b].item()) == rem[0]
    gm, gc = mask0.reshape(B, -1, cfg.bs), commit_g.reshape(B, -1, cfg.bs)
    assert np.all((gc.sum(-1) >= 1) == (gm.sum(-1) >= 1)) and np.all(commit_g <= mask0)
    x_g = x.cpu().numpy()
    assert np.array_equal(x_g[commit_g == 0], x0[commit_g == 0])
    assert np.array_equal(x_g[commit_g == 1], tok_g[commit_g == 1])
    assert np.array_equal(mask.cpu().numpy(), mask0 - commit_g)


# --------------------------------------------------------------------------------------------------------- #
# Whole blocks at full size, driven the way the benchmark drives them, in lock-step with the oracle on a
# subset of the batch (sequences are independent and keyed one by one, so the oracle's results for the
# subset are what the GPU must produce for those sequences inside the full batch).
# --------------------------------------------------------------------------------------------------------- #
def lockstep_block_fullsize(name, block, seqs, max_excluded=0.05):
    """The GPU runs ALL sequences of workload `name` through one whole block with GpuRollout.step exactly as
    the benchmark's loop queues it: the LM-head row bound is the still-masked total of two steps ago (the
    one-step-late poll), M_expected guesses the count from it, sequences that finished are skipped by the
    attention call (seq_active) and written back inside the selection's launch (DLM_WB_WHILE_ACTIVE); for the
    top-k workload the exact row schedule replaces the late bound.  OracleRollout runs `seqs` beside it; every
    step both start from the same state, and after a step the oracle marks numerically ambiguous it is
    re-synchronised to the GPU's state (same rules as tests/test_gpu_rollout.py::lockstep)."""
    cfg = synth.CONFIGS[name]
    seqs = list(seqs)
    B, Lb = cfg.B, cfg.Lb
    w = synth.w_vocab(cfg)
    o = oracle.OracleRollout(cfg, synth, seqs=seqs, w=w)
    g = GpuRollout(cfg, bf16_dev(w), DEV, record_steps=True)
    g.late_bound = True
    k0, v0 = synth.cache_kv(cfg, 0)
    g.cache_k.copy_(bf16_dev(k0))
    g.cache_v.copy_(bf16_dev(v0))
    del k0, v0
    x0 = synth.initial_tokens(cfg, cfg.L)
    g.x.copy_(dev(x0))
    o.begin_block(block)
    rk = rv = None
    if cfg.refresh and block > 0:
        k, v = synth.cache_kv(cfg, block)
        rk, rv = bf16_dev(k), bf16_dev(v)
        del k, v
    g.begin_block(block, refresh_k=rk, refresh_v=rv)      # every position masked, as in the benchmark
    torch.cuda.synchronize()
    P = o.P
    assert np.array_equal(bf16_host(g.cache_k[seqs]), o.cache_k) and np.array_equal(bf16_host(g.cache_v[seqs]), o.cache_v)
    cache_start = (bf16_host(g.cache_k), bf16_host(g.cache_v))
    outside = np.ones(cfg.L, bool)
    outside[P:P + Lb] = False
    stats = dict(steps=0, seq_steps=0, excluded=0, oracle_rows=0, worst_attn=0.0, worst_conf=0.0, bounds=[])
    rem_hist = []                    # still-masked total after every step (what the benchmark's poll reads)
    mask_prev = np.ones((B, Lb), np.uint8)
    x_prev = x0.copy()
    final_kv = {}
    step = 0
    worst = None
    while mask_prev.any():
        assert step <= Lb, "block did not finish"
        if step >= 2:
            g.set_row_bound(rem_hist[step - 2] if rem_hist[step - 2] > 0 else 1)
        stats["bounds"].append(g.m_host if not g._exact_rows else -1)
        q = synth.step_q(cfg, block, step)
        kb, vb = synth.step_kv(cfg, block, step)
        hid = synth.step_hidden(cfg, block, step)
        r = o.step() if o.mask.any() else None
        g.step(bf16_dev(q), bf16_dev(kb), bf16_dev(vb), bf16_dev(hid))
        torch.cuda.synchronize()
        commit_g = g.commit_now.cpu().numpy()
        x_g, mask_g = g.x.cpu().numpy(), g.mask.cpu().numpy()
        conf_all, tok_all = g.conf.cpu().numpy(), g.tok.cpu().numpy()
        n_commit_g, remaining_g = g.n_commit.cpu().numpy(), g.remaining.cpu().numpy()
        # ---- properties of the whole batch --------------------------------------------------------------
        had = mask_prev.sum(axis=1) > 0
        assert np.all(n_commit_g[had] >= 1) and np.all(n_commit_g[~had] == 0)
        assert np.array_equal(remaining_g, mask_g.sum(axis=1)) and np.all(mask_g <= mask_prev)
        assert np.array_equal(commit_g, mask_prev - mask_g)
        cm = commit_g.astype(bool)
        blk = x_g[:, P:P + Lb]
        assert np.array_equal(blk[cm], tok_all[cm]) and np.array_equal(blk[~cm], x_prev[:, P:P + Lb][~cm])
        assert np.array_equal(x_g[:, outside], x0[:, outside])
        assert np.all((tok_all[mask_prev.astype(bool)] >= 0) & (tok_all[mask_prev.astype(bool)] < cfg.V - 1))
        if cfg.rule == "topk":
            assert np.all(n_commit_g[had] == np.minimum(cfg.k, mask_prev.sum(axis=1)[had]))
        # selection is exact given the confidences the GPU produced, for every sequence of the batch
        commit_ref, nc_ref, rem_ref = select_commit(conf_all.astype(np.float64), mask_prev, rule=cfg.rule,
                                                    tau=float(np.float32(cfg.tau)), k=cfg.k)
        assert np.array_equal(commit_g, commit_ref) and np.array_equal(n_commit_g, nc_ref)
        flat = np.flatnonzero(mask_g.ravel())
        assert int(g.m_dev.item()) == len(flat) and np.array_equal(g.row_idx.cpu().numpy()[:len(flat)], flat)
        # cache: a sequence that finished holds its final step's block K/V; everything outside the slot is untouched
        ck_g, cv_g = bf16_host(g.cache_k), bf16_host(g.cache_v)
        for s in range(B):
            if remaining_g[s] == 0 and n_commit_g[s] > 0:
                final_kv[s] = (kb[s].copy(), vb[s].copy())
            if s in final_kv:
                assert np.array_equal(ck_g[s, :, P:P + Lb], final_kv[s][0]), f"K write-back, seq {s}"
                assert np.array_equal(cv_g[s, :, P:P + Lb], final_kv[s][1]), f"V write-back, seq {s}"
        assert np.array_equal(ck_g[:, :, outside], cache_start[0][:, :, outside])
        assert np.array_equal(cv_g[:, :, outside], cache_start[1][:, :, outside])
        # ---- the oracle's sequences, element by element -------------------------------------------------
        if r is not None:
            mb = r["mask_before"]
            assert np.array_equal(mb, mask_prev[seqs])
            O_g = bf16_host(g.O)[seqs]
            act = mb.any(axis=1) if step > 0 else np.ones(len(seqs), bool)
            rep = attn_err_report(O_g[act], r["O"][act])
            if worst is None or rep["rms_floor"] > worst["rms_floor"]:
                worst = rep
            assert rep["rms_floor"] <= ATTN_TOL, f"step {step}: attention {fmt_err(rep)}"
            lse_g = g.lse_attn.cpu().numpy()[seqs]
            assert np.abs(lse_g[act] - r["lse_attn"][act]).max() <= 2e-3
            rows = r["row_idx"]
            stats["oracle_rows"] += len(rows)
            conf_g = conf_all[seqs].ravel()[rows].astype(np.float64)
            tok_g = tok_all[seqs].ravel()[rows]
            lm = r["lm"]
            cerr = float(np.abs(conf_g - lm["conf"]).max())
            stats["worst_conf"] = max(stats["worst_conf"], cerr)
            assert cerr <= CONF_TOL, f"step {step}: confidence abs err {cerr}"
            clear_tok = (lm["zmax"] - lm["z2nd"]) >= NEAR
            assert np.array_equal(tok_g[clear_tok], lm["tok"][clear_tok])
            assert np.abs(g.lse.cpu().numpy().reshape(B, Lb)[seqs].ravel()[rows] - lm["lse"]).max() <= 5e-3   # logits-scale, fp32 sums over Dh = 4096
            conf_o = r["conf"]
            for n, s in enumerate(seqs):
                if not mb[n].any():
                    assert not commit_g[s].any()
                    continue
                stats["seq_steps"] += 1
                m = mb[n].astype(bool)
                top = np.sort(conf_o[n][m])[::-1]
                if cfg.rule == "threshold":
                    amb = bool((np.abs(conf_o[n][m] - cfg.tau) < NEAR).any())
                    amb |= bool(len(top) > 1 and top[0] - top[1] < NEAR and top[0] < cfg.tau + NEAR)
                else:
                    kk = min(cfg.k, len(top))
                    amb = bool(len(top) > kk and top[kk - 1] - top[kk] < NEAR)
                sel = r["commit"][n].astype(bool)
                amb_tok = bool((~clear_tok[(rows // Lb) == n]).any())
                if np.array_equal(commit_g[s], r["commit"][n]):
                    same_tok = np.array_equal(x_g[s, P:P + Lb][sel], r["tok"][n][sel])
                    assert same_tok or amb_tok, f"token mismatch, step {step} seq {s}"
                    stats["excluded"] += 0 if same_tok else 1
                else:
                    assert amb, f"commit mask mismatch, step {step} seq {s}"
                    stats["excluded"] += 1
            # both sides start the next step from the same state (a no-op unless an ambiguous step differed)
            o.x[:] = x_g[seqs]
            o.mask[:] = mask_g[seqs]
            o.cache_k[:] = ck_g[seqs]
            o.cache_v[:] = cv_g[seqs]
        rem_hist.append(int(remaining_g.sum()))
        mask_prev, x_prev = mask_g, x_g
        stats["steps"] += 1
        step += 1
    assert not o.mask.any() and set(final_kv) == set(range(B))
    # the step the one-step-late poll queues after the block has finished finds nothing masked and changes nothing
    g.set_row_bound(rem_hist[-2] if len(rem_hist) >= 2 and rem_hist[-2] > 0 else 1)
    kb, vb = synth.step_kv(cfg, block, step)
    g.step(bf16_dev(synth.step_q(cfg, block, step)), bf16_dev(kb), bf16_dev(vb), bf16_dev(synth.step_hidden(cfg, block, step)))
    torch.cuda.synchronize()
    assert np.array_equal(g.x.cpu().numpy(), x_prev) and not g.mask.any().item() and int(g.m_dev.item()) == 0
    assert not g.commit_now.any().item() and not g.n_commit.any().item()
    assert np.array_equal(bf16_host(g.cache_k), ck_g) and np.array_equal(bf16_host(g.cache_v), cv_g)
    assert stats["excluded"] <= max_excluded * max(1, stats["seq_steps"]), stats
    stats["worst_attn"] = worst
    print(f"{name} block {block} seqs {seqs}: {stats['steps']} steps, {stats['seq_steps']} oracle sequence-steps "
          f"({stats['excluded']} excluded as ambiguous), {stats['oracle_rows']} LM-head rows checked, worst confidence "
          f"error {stats['worst_conf']:.2e}, worst attention step: {fmt_err(worst)}; row bounds {stats['bounds']}", flush=True)
    return stats


def test_c2_whole_block_lockstep_as_the_benchmark_drives_it():
    st = lockstep_block_fullsize("c2", block=3, seqs=[0, 5])
    assert st["steps"] >= 4


def test_c3_whole_block_lockstep_as_the_benchmark_drives_it():
    lockstep_block_fullsize("c3", block=9, seqs=[2, 15])


def test_c4_whole_block_lockstep_as_the_benchmark_drives_it():
    st = lockstep_block_fullsize("c4", block=2, seqs=[0, 31])
    assert st["steps"] == 8


def test_c5a_whole_block_lockstep_as_the_benchmark_drives_it():
    lockstep_block_fullsize("c5a", block=0, seqs=[0, 1, 62, 63])
