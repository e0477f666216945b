"""Invariants of the oracle's rollout loop and full-sequence pass (CPU only)."""
import numpy as np
import pytest

import oracle
from oracle import KV
from paper_2604_04215_amd import synth


def _check_invariants(cfg, seqs=None):
    ro = oracle.OracleRollout(cfg, synth, seqs=seqs)
    n = len(ro.seqs)
    x0 = ro.x.copy()
    committed_pos = np.zeros((n, cfg.L), bool)
    seen = {"steps": 0}

    def on_step(r, out):
        mb, ma = out["mask_before"], r.mask
        had = mb.sum(axis=1) > 0
        # every sequence that still has masked positions commits at least one
        assert np.all(out["n_commit"][had] >= 1) and np.all(out["n_commit"][~had] == 0)
        # the masked count strictly decreases and nothing gets re-masked
        assert np.all(ma.sum(axis=1)[had] < mb.sum(axis=1)[had]) and np.all(ma <= mb)
        assert np.array_equal(out["remaining"], ma.sum(axis=1))
        # committed tokens never change; uncommitted positions keep their old content
        P = r.P
        now = np.zeros_like(committed_pos)
        now[:, P:P + cfg.Lb] = out["commit"].astype(bool)
        assert not (now & committed_pos).any()
        assert np.array_equal(r.x[committed_pos], seen["x"][committed_pos]) if "x" in seen else True
        assert np.array_equal(r.x[now], out["tok"][out["commit"].astype(bool)])
        untouched = ~(now | committed_pos)
        assert np.array_equal(r.x[untouched], x0[untouched])
        committed_pos[:] |= now
        seen["x"] = r.x.copy()
        # predictions never produce the stand-in <MASK> id
        assert np.all(out["lm"]["tok"] != cfg.forbid_token)
        seen["steps"] += 1

    res = ro.run(on_step=on_step)
    n_init = cfg.init_masked if cfg.init_masked is not None else cfg.Lb
    assert res["committed"] == n * (n_init + (cfg.n_blocks - 1) * cfg.Lb if cfg.init_masked is not None
                                    else cfg.n_blocks * cfg.Lb)
    assert not ro.mask.any()
    return ro, res


@pytest.mark.parametrize("name", ["mini1", "mini2", "mini3", "mini4", "mini5a"])
def test_rollout_invariants(name):
    cfg = synth.CONFIGS[name]
    ro, res = _check_invariants(cfg)
    if cfg.rule == "topk":
        assert res["steps"] == [cfg.Lb // cfg.k] * cfg.n_blocks       # fixed schedule: exactly Lb/k steps
    else:
        assert all(1 <= s <= cfg.Lb for s in res["steps"])


def test_std_reading_commits_one_per_step():
    # W ~ N(0, std Dh^-1/2): logits ~ N(0,1), confidences tiny, the threshold never fires
    cfg = synth.CONFIGS["mini2"].replace(w_dist="std", gen=32)
    ro, res = _check_invariants(cfg)
    assert res["steps"] == [32]


def test_sequences_are_independent_of_batch():
    cfg = synth.CONFIGS["mini3"]
    full = oracle.OracleRollout(cfg, synth)
    full.run(blocks=[0, 1])
    sub = oracle.OracleRollout(cfg, synth, seqs=[2])
    sub.run(blocks=[0, 1])
    assert np.array_equal(full.x[2], sub.x[0])
    assert np.array_equal(full.cache_k[2], sub.cache_k[0])


def test_stop_copy_resume_gives_same_trajectory():
    cfg = synth.CONFIGS["mini2"]
    a = oracle.OracleRollout(cfg, synth)
    a.begin_block(0)
    a.step(); a.step()
    b = oracle.OracleRollout(cfg, synth)
    b.restore(a.snapshot())
    while a.mask.any():
        a.step()
    while b.mask.any():
        b.step()
    assert np.array_equal(a.x, b.x) and a.step_idx == b.step_idx


def test_writeback_and_refresh():
    cfg = synth.CONFIGS["mini2"]
    ro = oracle.OracleRollout(cfg, synth)
    k0, v0 = synth.cache_kv(cfg, 0)
    ro.begin_block(0)
    last_kv = {}
    while ro.mask.any():
        before = ro.mask.sum(axis=1)
        step = ro.step_idx
        out = ro.step()
        for b in range(cfg.B):
            if before[b] > 0 and out["remaining"][b] == 0:
                last_kv[b] = step
    P, Lb = cfg.prompt, cfg.Lb
    for b in range(cfg.B):
        kb, vb = synth.step_kv(cfg, 0, last_kv[b], seqs=[b])
        assert np.array_equal(ro.cache_k[b, :, P:P + Lb], kb[0])
        assert np.array_equal(ro.cache_v[b, :, P:P + Lb], vb[0])
    assert np.array_equal(ro.cache_k[:, :, :P], k0[:, :, :P])
    assert np.array_equal(ro.cache_k[:, :, P + Lb:], k0[:, :, P + Lb:])
    # refresh at the next block installs the new image on the prefix (incl. the block just done)
    ro.begin_block(1)
    k1, _ = synth.cache_kv(cfg, 1)
    assert np.array_equal(ro.cache_k[:, :, :P + Lb], k1[:, :, :P + Lb])
    assert np.array_equal(ro.cache_k[:, :, P + Lb:], k0[:, :, P + Lb:])       # prefix-only cache


def test_dual_cache_sees_suffix_and_prefix_only_does_not():
    cfg = synth.CONFIGS["mini3"]
    ro = oracle.OracleRollout(cfg, synth)
    ro.begin_block(1)
    assert ro.S == cfg.L - ro.P - cfg.Lb and ro.S > 0
    kb, vb = synth.step_kv(cfg, 1, 0)
    segs = ro.segments(kb, vb)
    assert [s.len for s in segs] == [ro.P, cfg.Lb, ro.S] and [s.pos0 for s in segs] == [0, ro.P, ro.P + cfg.Lb]
    ro2 = oracle.OracleRollout(synth.CONFIGS["mini2"], synth)
    ro2.begin_block(0)
    assert ro2.S == 0


def test_full_pass_block_causal():
    cfg = synth.FULLPASS["mini5b"]
    out = oracle.full_pass(cfg, synth)
    mask0, commit = out["mask_before"], out["commit"]
    B, L, bs = cfg.B, cfg.L, cfg.bs
    g = mask0.reshape(B, L // bs, bs)
    cg = commit.reshape(B, L // bs, bs)
    # every block with a masked position commits at least one; blocks without commit nothing
    assert np.all((cg.sum(-1) >= 1) == (g.sum(-1) >= 1))
    assert np.all(commit <= mask0)
    assert np.array_equal(out["x"][commit == 0], out["x_before"][commit == 0])
    assert np.array_equal(out["x"][commit == 1], out["tok"][commit == 1])
    assert np.array_equal(out["remaining"], (mask0 - commit).sum(axis=1))
    # the rollout call on block j with the exact cache reproduces rows of the full pass
    q, k, v = synth.fullpass_qkv(cfg)
    P = 100
    Or, _ = oracle.attention(q[:, P:P + bs], [KV(k[:, :, :P], v[:, :, :P], 0), KV(k[:, :, P:P + bs], v[:, :, P:P + bs], P)],
                             mask_mode="block_causal", bs=bs, q_pos0=P)
    assert np.allclose(out["O"][:, P:P + bs], Or, atol=1e-13)
