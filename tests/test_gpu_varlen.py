"""Packed variable-length attention (cu_seqlens mode of dlm_block_attn) against the oracle (GPU)."""
import numpy as np
import pytest
import torch

import oracle
from oracle import KV
from paper_2604_04215_amd import binding as dlm
from paper_2604_04215_amd import synth
from gpu_util import DEV, attn_rel_err, bf16_dev, bf16_host, dev, rnd

pytestmark = pytest.mark.gpu

TOL = 2e-2
LSE_TOL = 2e-3


def run_varlen(lens, Hq, Hkv, d, mode="full", bs=0, variant=0, seed=0, max_seqlen=None, pad_rows=0):
    lens = np.asarray(lens, np.int64)
    T = int(lens.sum())
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    q, k, v = rnd(seed + 1, (T, Hq, d)), rnd(seed + 2, (T, Hkv, d)), rnd(seed + 3, (T, Hkv, d))
    ref, ref_lse = oracle.attention_varlen(q, k, v, cu, mask_mode=mode, bs=bs)
    # K and V are column slices of one fused [T, 2, Hkv, d] buffer: token stride differs from Hkv * d
    kv = torch.empty((T + pad_rows, 2, Hkv, d), dtype=torch.bfloat16, device=DEV)
    kv[:T, 0], kv[:T, 1] = bf16_dev(k), bf16_dev(v)
    qd = bf16_dev(q)
    out = torch.full((T, Hq, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    lse = torch.full((Hq, T), float("nan"), dtype=torch.float32, device=DEV)
    mx = int(lens.max()) if max_seqlen is None else max_seqlen
    dlm.set_option("attn_variant", variant)
    try:
        dlm.varlen_attn(qd, kv[:T, 0], kv[:T, 1], out, dev(cu), mx,
                        mask_mode=dlm.MASK_BLOCK_CAUSAL if mode == "block_causal" else dlm.MASK_FULL,
                        block_size=bs, lse=lse)
        torch.cuda.synchronize()
    finally:
        dlm.set_option("attn_variant", 0)
    if T == 0:
        return
    err = attn_rel_err(bf16_host(out), ref)
    assert err <= TOL, f"varlen attention rel err {err}"
    assert np.abs(lse.cpu().numpy().astype(np.float64) - ref_lse).max() <= LSE_TOL


@pytest.mark.parametrize("variant", [0, 2, 3, 4, 5, 6, 7, 11])
def test_ragged_mix_row_split_shapes(variant):
    # lengths around the 32-key tile and the 128-row workgroup, an empty sequence, one-token sequences
    run_varlen([1, 31, 32, 33, 200, 0, 129, 1, 257], Hq=4, Hkv=2, d=128, variant=variant, seed=10)


@pytest.mark.parametrize("d,Hq,Hkv", [(64, 4, 4), (64, 6, 2), (128, 8, 1)])
def test_head_layouts(d, Hq, Hkv):
    run_varlen([70, 5, 130, 64], Hq=Hq, Hkv=Hkv, d=d, seed=20)


def test_short_sequences_use_key_split_shape():
    # g * max_seqlen <= 32 rows per KV head: the key-split kernel shape serves the packed batch too
    run_varlen([32, 7, 0, 19, 32, 1], Hq=2, Hkv=2, d=128, seed=30)
    run_varlen([8, 3, 5], Hq=8, Hkv=2, d=64, seed=31)


@pytest.mark.parametrize("bs", [4, 32])
def test_block_causal_positions_restart_per_sequence(bs):
    run_varlen([67, 128, 9, 200], Hq=4, Hkv=2, d=128, mode="block_causal", bs=bs, seed=40)


def test_loose_upper_bound_on_length_and_empty_batch():
    run_varlen([50, 90, 10], Hq=4, Hkv=4, d=64, max_seqlen=256, seed=50)     # bound above the longest sequence
    run_varlen([0, 0], Hq=4, Hkv=4, d=64, max_seqlen=16, seed=51, pad_rows=1)


def test_truncation_to_the_stated_bound():
    # a sequence longer than Lq is cut to its first Lq tokens (queries and keys); the rest is left untouched
    lens, Hq, Hkv, d, cap = [20, 100], 2, 2, 64, 64
    T = sum(lens)
    cu = np.array([0, 20, 120], np.int32)
    q, k, v = rnd(61, (T, Hq, d)), rnd(62, (T, Hkv, d)), rnd(63, (T, Hkv, d))
    out = torch.zeros((T, Hq, d), dtype=torch.bfloat16, device=DEV)
    dlm.varlen_attn(bf16_dev(q), bf16_dev(k), bf16_dev(v), out, dev(cu), cap)
    torch.cuda.synchronize()
    got = bf16_host(out)
    ref0, _ = oracle.attention_varlen(q[:20], k[:20], v[:20], [0, 20])
    ref1, _ = oracle.attention_varlen(q[20:20 + cap], k[20:20 + cap], v[20:20 + cap], [0, cap])
    assert attn_rel_err(got[:20], ref0) <= TOL and attn_rel_err(got[20:20 + cap], ref1) <= TOL
    assert not got[20 + cap:].any()


def test_rejects_a_bound_too_small_for_the_token_count():
    T, Hq, d = 64, 2, 64
    z = torch.zeros((T, Hq, d), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(dlm.DlmError):
        dlm.varlen_attn(z, z, z, z, dev(np.array([0, 64], np.int32)), 16)     # 64 tokens cannot fit B * Lq = 16


def test_full_size_packed_batch_sampled_rows():
    """The 128-sequence packed batch (about 64k tokens, 32 heads of 128): sampled rows against the oracle; every
    output row must have been written (no NaN from the initial fill survives)."""
    cfg = synth.VARLEN["v1"]
    q, k, v, cu = synth.varlen_qkv(cfg)
    T = int(cu[-1])
    out = torch.full((T, cfg.Hq, cfg.d), float("nan"), dtype=torch.bfloat16, device=DEV)
    lse = torch.full((cfg.Hq, T), float("nan"), dtype=torch.float32, device=DEV)
    print("inputs drawn", T, flush=True)
    dlm.varlen_attn(bf16_dev(q), bf16_dev(k), bf16_dev(v), out, dev(cu), int(np.diff(cu).max()), lse=lse)
    torch.cuda.synchronize()
    got, got_lse = bf16_host(out), lse.cpu().numpy()
    assert np.isfinite(got_lse).all() and np.isfinite(synth.bf16_bits_to_f32(got)).all()
    rng = np.random.default_rng(cfg.seed)
    for b in [0, cfg.B - 1, int(np.argmax(np.diff(cu))), int(np.argmin(np.diff(cu)))] + list(rng.integers(0, cfg.B, 4)):
        a, e = int(cu[b]), int(cu[b + 1])
        n = 6
        rows = np.stack([np.zeros(n, np.int64), rng.integers(0, cfg.Hq, n), rng.integers(0, e - a, n)], 1).astype(np.int32)
        rows[0, 2], rows[1, 2] = 0, e - a - 1
        seg = KV(np.ascontiguousarray(k[a:e].transpose(1, 0, 2))[None], np.ascontiguousarray(v[a:e].transpose(1, 0, 2))[None], 0)
        ref, ref_lse = oracle.attention(q[a:e][None], [seg], rows=rows)
        g = got[a + rows[:, 2], rows[:, 1]]
        assert attn_rel_err(g, ref) <= TOL
        assert np.abs(got_lse[rows[:, 1], a + rows[:, 2]] - ref_lse).max() <= LSE_TOL
