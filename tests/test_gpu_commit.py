"""dlm_unmask_commit / dlm_mask_compact / dlm_kv_refresh against the oracle (GPU, bit-exact)."""
import numpy as np
import pytest
import torch

from oracle.denoise import apply_commit, select_commit
from paper_2604_04215_amd import binding as dlm
from gpu_util import DEV, bf16_dev, bf16_host, dev, rnd

pytestmark = pytest.mark.gpu


def run_commit(conf, tok, mask, x, x_pos0, *, rule, tau=0.0, k=0, force=True, group_len=None, step=3,
               writeback=dlm.WB_NONE, src=None, cache=None, cache_pos0=0, active_in=None):
    B, n = mask.shape
    d_conf, d_tok = dev(conf.astype(np.float32)), dev(tok.astype(np.int32))
    big_mask = torch.zeros((B, n + 8), dtype=torch.uint8, device=DEV)        # strided view on purpose
    d_mask = big_mask[:, :n]
    d_mask.copy_(dev(mask))
    d_x = dev(x.copy())
    commit_now = torch.full((B, n), 9, dtype=torch.uint8, device=DEV)
    n_commit = torch.full((B,), -1, dtype=torch.int32, device=DEV)
    remaining = torch.full((B,), -1, dtype=torch.int32, device=DEV)
    row_idx = torch.full((B * n,), -1, dtype=torch.int32, device=DEV)
    next_m = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    cstep = torch.full((B, n), -1, dtype=torch.int16, device=DEV)
    kw = {}
    if writeback != dlm.WB_NONE:
        kw = dict(src_block=(src[0], src[1], 0), cache_k=cache[0], cache_v=cache[1], cache_pos0=cache_pos0)
        if active_in is not None:
            kw["active_in"] = dev(np.asarray(active_in, np.int32))
    dlm.unmask_commit(d_conf, d_tok, d_x, d_mask, n_commit, remaining, x_pos0=x_pos0, group_len=group_len,
                      rule=dlm.RULE_THRESHOLD if rule == "threshold" else dlm.RULE_TOPK, threshold=tau,
                      force_top1=force, k=k, commit_now=commit_now, next_row_idx=row_idx, next_m=next_m,
                      commit_step=cstep, step=step, writeback=writeback, **kw)
    torch.cuda.synchronize()
    assert float(big_mask[:, n:].sum()) == 0
    return dict(x=d_x.cpu().numpy(), mask=d_mask.cpu().numpy(), commit=commit_now.cpu().numpy(),
                n_commit=n_commit.cpu().numpy(), remaining=remaining.cpu().numpy(),
                row_idx=row_idx.cpu().numpy(), next_m=int(next_m.item()), cstep=cstep.cpu().numpy())


def check_against_oracle(conf, tok, mask, x, x_pos0, got, *, rule, tau=0.0, k=0, force=True, group_len=None, step=3):
    conf32 = conf.astype(np.float32)                       # the decision is taken on the fp32 values both sides see
    commit, n_commit, remaining = select_commit(conf32.astype(np.float64), mask, rule=rule,
                                                tau=float(np.float32(tau)), k=k, force_top1=force,
                                                group_len=group_len)
    x_ref, m_ref = x.copy(), mask.copy()
    apply_commit(x_ref, x_pos0, m_ref, tok, commit)
    assert np.array_equal(got["commit"], commit)
    assert np.array_equal(got["x"], x_ref) and np.array_equal(got["mask"], m_ref)
    assert np.array_equal(got["n_commit"], n_commit) and np.array_equal(got["remaining"], remaining)
    flat = np.flatnonzero(m_ref.ravel())
    assert got["next_m"] == len(flat) and np.array_equal(got["row_idx"][:len(flat)], flat)
    assert np.array_equal(got["cstep"], np.where(commit == 1, step, -1))


@pytest.mark.parametrize("rule,tau,k", [("threshold", 0.9, 0), ("threshold", 0.5, 0), ("threshold", 1.5, 0),
                                        ("threshold", 0.0, 0), ("topk", 0, 1), ("topk", 0, 4), ("topk", 0, 40)])
@pytest.mark.parametrize("B,n,group_len", [(8, 32, None), (3, 32, 4), (2, 200, 100), (2, 600, 300), (1, 1024, None),
                                           (5, 64, 1), (20, 200, None), (40, 512, None),
                                           (4, 64, 2), (4, 64, 8), (2, 30, 3), (70, 1000, 4),
                                           (16, 1024, None),     # the longest group, 16384 positions: largest one-workgroup problem
                                           (17, 1024, None),     # one sequence more: the wave-per-group path
                                           (15, 1023, None)])
def test_selection_bit_exact(rule, tau, k, B, n, group_len):
    import zlib
    rng = np.random.default_rng(zlib.crc32(repr((rule, tau, k, B, n, group_len)).encode()))
    conf = np.round(rng.random((B, n)), 2)                 # coarse grid: many ties, exact in fp32 compares
    conf[rng.random((B, n)) < 0.1] = 0.9                   # exactly at the threshold
    tok = rng.integers(0, 50000, size=(B, n))
    mask = (rng.random((B, n)) < 0.6).astype(np.uint8)
    mask[0, :] = 0 if B > 1 else mask[0, :]                # a finished sequence
    x = rng.integers(0, 50000, size=(B, n + 20)).astype(np.int32)
    got = run_commit(conf, tok, mask, x, 11, rule=rule, tau=tau, k=k, group_len=group_len)
    check_against_oracle(conf, tok, mask, x, 11, got, rule=rule, tau=tau, k=k, group_len=group_len)


def test_host_visible_total():
    """The single-workgroup path can publish the still-masked total straight into pinned host memory."""
    rng = np.random.default_rng(12)
    B, n = 8, 32
    conf, tok = rng.random((B, n)).astype(np.float32), rng.integers(0, 100, size=(B, n)).astype(np.int32)
    mask = (rng.random((B, n)) < 0.7).astype(np.uint8)
    d_mask, d_x = dev(mask), torch.zeros((B, n), dtype=torch.int32, device=DEV)
    n_commit = torch.zeros(B, dtype=torch.int32, device=DEV)
    remaining = torch.zeros(B, dtype=torch.int32, device=DEV)
    host = torch.full((1,), -5, dtype=torch.int32).pin_memory()
    dlm.unmask_commit(dev(conf), dev(tok), d_x, d_mask, n_commit, remaining, x_pos0=0, rule=dlm.RULE_TOPK, k=3,
                      host_remaining_total=host)
    torch.cuda.synchronize()
    assert int(host[0]) == int(remaining.sum().item()) == int(d_mask.sum().item())
    # not available when the multi-kernel path is needed
    with pytest.raises(dlm.DlmError):
        dlm.unmask_commit(dev(conf), dev(tok), d_x, d_mask, n_commit, remaining, x_pos0=0, group_len=4,
                          rule=dlm.RULE_TOPK, k=1, host_remaining_total=host)


def test_host_visible_maximum():
    """Beside the total, the most positions any one sequence still has masked (what tells a late-polling host that the next
    step ends the block): after every step of a small rollout-like sequence of commits."""
    rng = np.random.default_rng(13)
    B, n = 20, 32
    mask = (rng.random((B, n)) < 0.8).astype(np.uint8)
    mask[3] = 0
    d_mask, d_x = dev(mask), torch.zeros((B, n), dtype=torch.int32, device=DEV)
    n_commit = torch.zeros(B, dtype=torch.int32, device=DEV)
    remaining = torch.zeros(B, dtype=torch.int32, device=DEV)
    host = torch.full((1,), -5, dtype=torch.int32).pin_memory()
    host_max = torch.full((1,), -5, dtype=torch.int32).pin_memory()
    for step in range(40):
        conf, tok = rng.random((B, n)).astype(np.float32), rng.integers(0, 100, size=(B, n)).astype(np.int32)
        dlm.unmask_commit(dev(conf), dev(tok), d_x, d_mask, n_commit, remaining, x_pos0=0, rule=dlm.RULE_THRESHOLD,
                          threshold=0.8, force_top1=True, host_remaining_total=host, host_remaining_max=host_max)
        torch.cuda.synchronize()
        per_seq = d_mask.sum(1).cpu().numpy()
        assert int(host[0]) == int(per_seq.sum()) and int(host_max[0]) == int(per_seq.max())
        if per_seq.max() == 0:
            break
    assert per_seq.max() == 0
    with pytest.raises(dlm.DlmError):       # the maximum goes with the total
        dlm.unmask_commit(dev(conf), dev(tok), d_x, d_mask, n_commit, remaining, x_pos0=0, rule=dlm.RULE_TOPK, k=1,
                          host_remaining_max=host_max)


def test_no_forced_pick():
    rng = np.random.default_rng(3)
    conf, tok = rng.random((4, 32)) * 0.5, rng.integers(0, 100, size=(4, 32))
    mask = np.ones((4, 32), np.uint8)
    x = np.zeros((4, 32), np.int32)
    got = run_commit(conf, tok, mask, x, 0, rule="threshold", tau=0.9, force=False)
    check_against_oracle(conf, tok, mask, x, 0, got, rule="threshold", tau=0.9, force=False)
    assert got["n_commit"].sum() == 0


def test_full_pass_sized_groups():
    # 64 sequences x 4096 positions in groups of 4 with Bernoulli(0.5) masking
    rng = np.random.default_rng(4)
    B, n = 64, 4096
    conf = rng.random((B, n)).astype(np.float32)
    tok = rng.integers(0, 157183, size=(B, n))
    mask = (rng.random((B, n)) < 0.5).astype(np.uint8)
    x = rng.integers(0, 1000, size=(B, n)).astype(np.int32)
    got = run_commit(conf, tok, mask, x, 0, rule="threshold", tau=0.95, group_len=4)
    # the pure-Python oracle rule on a sample of sequences, properties on all
    for b in (0, 17, 63):
        check = run_commit  # noqa
        commit, n_commit, remaining = select_commit(conf[b:b + 1].astype(np.float64), mask[b:b + 1], rule="threshold",
                                                    tau=float(np.float32(0.95)), group_len=4)
        assert np.array_equal(got["commit"][b:b + 1], commit)
        assert got["n_commit"][b] == n_commit[0] and got["remaining"][b] == remaining[0]
    g_mask, g_commit = mask.reshape(B, -1, 4), got["commit"].reshape(B, -1, 4)
    assert np.all((g_commit.sum(-1) >= 1) == (g_mask.sum(-1) >= 1)) and np.all(got["commit"] <= mask)
    assert np.array_equal(got["x"][got["commit"] == 0], x[got["commit"] == 0])
    assert np.array_equal(got["x"][got["commit"] == 1], tok[got["commit"] == 1])
    assert got["next_m"] == int(got["mask"].sum())
    assert np.array_equal(got["row_idx"][:got["next_m"]], np.flatnonzero(got["mask"].ravel()))


@pytest.mark.parametrize("mode", [dlm.WB_BLOCK_WHEN_DONE, dlm.WB_COMMITTED_ROWS])
def test_writeback(mode):
    B, Hkv, Lb, d, L, P = 3, 2, 32, 128, 100, 40
    rng = np.random.default_rng(5)
    src_k, src_v = rnd(1, (B, Hkv, Lb, d)), rnd(2, (B, Hkv, Lb, d))
    c_k, c_v = rnd(3, (B, Hkv, L, d)), rnd(4, (B, Hkv, L, d))
    conf = rng.random((B, Lb))
    conf[0] = 0.99                                   # sequence 0 finishes in this call
    mask = np.ones((B, Lb), np.uint8)
    mask[2] = 0                                      # sequence 2 had finished earlier: no write-back
    tok = rng.integers(0, 100, size=(B, Lb))
    x = np.zeros((B, L), np.int32)
    dk, dv = bf16_dev(c_k), bf16_dev(c_v)
    got = run_commit(conf, tok, mask, x, P, rule="threshold", tau=0.9, writeback=mode,
                     src=(bf16_dev(src_k), bf16_dev(src_v)), cache=(dk, dv), cache_pos0=P)
    check_against_oracle(conf, tok, mask, x, P, got, rule="threshold", tau=0.9)
    want_k, want_v = c_k.copy(), c_v.copy()
    for b in range(B):
        for i in range(Lb):
            if (mode == dlm.WB_BLOCK_WHEN_DONE and got["remaining"][b] == 0 and got["n_commit"][b] > 0) or \
               (mode == dlm.WB_COMMITTED_ROWS and got["commit"][b, i]):
                want_k[b, :, P + i] = src_k[b, :, i]
                want_v[b, :, P + i] = src_v[b, :, i]
    assert np.array_equal(bf16_host(dk), want_k) and np.array_equal(bf16_host(dv), want_v)
    assert not np.array_equal(want_k, c_k)


@pytest.mark.parametrize("B,Hkv,Lb,d,group_len", [(5, 2, 32, 128, None), (3, 3, 40, 64, None), (2, 1, 700, 64, None),
                                                   (40, 2, 512, 64, None), (6, 2, 64, 128, 4)])
def test_writeback_while_active(B, Hkv, Lb, d, group_len):
    """Sequences flagged by active_in get the whole block copied, the others keep their cache rows, whatever this
    call's selection does; rows outside [P, P + Lb) are untouched.  Covers the copy inside the single-workgroup
    launch (first three), and the separate copy launch (more than 16384 positions; several groups per sequence)."""
    L, P = Lb + 50, 37
    rng = np.random.default_rng(Lb)
    src_k, src_v = rnd(21, (B, Hkv, Lb, d)), rnd(22, (B, Hkv, Lb, d))
    c_k, c_v = rnd(23, (B, Hkv, L, d)), rnd(24, (B, Hkv, L, d))
    conf = rng.random((B, Lb))
    conf[0] = 0.99
    mask = (rng.random((B, Lb)) < 0.6).astype(np.uint8)
    mask[-1] = 0
    active = (np.arange(B) % 3 != 1).astype(np.int32) * 7      # deliberately not derived from the mask
    tok = rng.integers(0, 100, size=(B, Lb))
    x = np.zeros((B, L), np.int32)
    dk, dv = bf16_dev(c_k), bf16_dev(c_v)
    got = run_commit(conf, tok, mask, x, P, rule="threshold", tau=0.9, group_len=group_len, writeback=dlm.WB_WHILE_ACTIVE,
                     src=(bf16_dev(src_k), bf16_dev(src_v)), cache=(dk, dv), cache_pos0=P, active_in=active)
    check_against_oracle(conf, tok, mask, x, P, got, rule="threshold", tau=0.9, group_len=group_len)
    want_k, want_v = c_k.copy(), c_v.copy()
    for b in range(B):
        if active[b]:
            want_k[b, :, P:P + Lb] = src_k[b]
            want_v[b, :, P:P + Lb] = src_v[b]
    assert np.array_equal(bf16_host(dk), want_k) and np.array_equal(bf16_host(dv), want_v)


def test_writeback_while_active_rejects_aliased_or_missing_counts():
    B, Hkv, Lb, d = 2, 1, 32, 64
    z = torch.zeros((B, Lb), device=DEV)
    conf, tok = z.float(), z.int()
    x, mask = torch.zeros((B, 64), dtype=torch.int32, device=DEV), torch.ones((B, Lb), dtype=torch.uint8, device=DEV)
    n_commit, remaining = torch.zeros(B, dtype=torch.int32, device=DEV), torch.zeros(B, dtype=torch.int32, device=DEV)
    src = torch.zeros((B, Hkv, Lb, d), dtype=torch.bfloat16, device=DEV)
    cache = torch.zeros((B, Hkv, 64, d), dtype=torch.bfloat16, device=DEV)
    kw = dict(x_pos0=0, rule=dlm.RULE_THRESHOLD, threshold=2.0, writeback=dlm.WB_WHILE_ACTIVE, src_block=(src, src, 0),
              cache_k=cache, cache_v=cache, cache_pos0=0)
    for bad in (None, remaining, n_commit):
        with pytest.raises(dlm.DlmError):
            dlm.unmask_commit(conf, tok, x, mask, n_commit, remaining, active_in=bad, **kw)
    torch.cuda.synchronize()
    assert int(mask.sum()) == B * Lb and float(cache.float().abs().sum()) == 0    # nothing ran


def test_kv_refresh_bitwise_and_strided():
    B, Hkv, L, d = 2, 3, 150, 128
    img_k, img_v = rnd(11, (B, Hkv, L, d)), rnd(12, (B, Hkv, L, d))
    old_k, old_v = rnd(13, (B, Hkv, L, d)), rnd(14, (B, Hkv, L, d))
    ik, iv, ck, cv = bf16_dev(img_k), bf16_dev(img_v), bf16_dev(old_k), bf16_dev(old_v)
    P, Lb = 70, 32
    dlm.kv_refresh(ik[:, :, :P], iv[:, :, :P], ck, cv, 0)
    dlm.kv_refresh(ik[:, :, P + Lb:], iv[:, :, P + Lb:], ck, cv, P + Lb)
    torch.cuda.synchronize()
    want_k, want_v = img_k.copy(), img_v.copy()
    want_k[:, :, P:P + Lb], want_v[:, :, P:P + Lb] = old_k[:, :, P:P + Lb], old_v[:, :, P:P + Lb]
    assert np.array_equal(bf16_host(ck), want_k) and np.array_equal(bf16_host(cv), want_v)
    with pytest.raises(ValueError):
        dlm.kv_refresh(ik, iv, ck, cv, 1)


def test_mask_compact():
    rng = np.random.default_rng(6)
    for B, n in [(8, 32), (3, 700), (1, 5000), (2, 1)]:
        mask = (rng.random((B, n)) < 0.4).astype(np.uint8)
        d_mask = dev(mask)
        row_idx = torch.full((B * n,), -1, dtype=torch.int32, device=DEV)
        m = torch.zeros(1, dtype=torch.int32, device=DEV)
        dlm.mask_compact(d_mask, row_idx, m)
        torch.cuda.synchronize()
        flat = np.flatnonzero(mask.ravel())
        assert int(m.item()) == len(flat) and np.array_equal(row_idx.cpu().numpy()[:len(flat)], flat)
