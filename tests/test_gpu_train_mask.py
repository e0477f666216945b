"""Block-diffusion training attention (per-segment block rules of dlm_block_attn) against the oracle (GPU)."""
import numpy as np
import pytest
import torch

import oracle
from oracle import KV
from paper_2604_04215_amd import binding as dlm
from paper_2604_04215_amd import synth
from gpu_util import DEV, attn_rel_err, bf16_dev, bf16_host, rnd

pytestmark = pytest.mark.gpu

TOL, LSE_TOL = 2e-2, 2e-3


def gpu_train_attention(qn, kn, vn, qc, kc, vc, bs, variant=0):
    B, L, Hq, d = qn.shape
    qn_d, kn_d, vn_d, qc_d, kc_d, vc_d = (bf16_dev(a) for a in (qn, kn, vn, qc, kc, vc))
    On = torch.full((B, L, Hq, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    Oc = torch.full_like(On, float("nan"))
    Ln = torch.full((B, Hq, L), float("nan"), dtype=torch.float32, device=DEV)
    Lc = torch.full_like(Ln, float("nan"))
    dlm.set_option("attn_variant", variant)
    try:
        dlm.block_attn(qn_d, On, prefix=(kc_d, vc_d, 0, dlm.SEG_EARLIER_BLOCKS), block=(kn_d, vn_d, 0, dlm.SEG_SAME_BLOCK),
                       mask_mode=dlm.MASK_BLOCK_CAUSAL, block_size=bs, q_pos0=0, lse=Ln)
        dlm.block_attn(qc_d, Oc, block=(kc_d, vc_d, 0, dlm.SEG_CAUSAL), mask_mode=dlm.MASK_BLOCK_CAUSAL,
                       block_size=bs, q_pos0=0, lse=Lc)
        torch.cuda.synchronize()
    finally:
        dlm.set_option("attn_variant", 0)
    return bf16_host(On), Ln.cpu().numpy().astype(np.float64), bf16_host(Oc), Lc.cpu().numpy().astype(np.float64)


def make(B, L, Hq, Hkv, d, seed):
    return (rnd(seed + 1, (B, L, Hq, d)), rnd(seed + 2, (B, Hkv, L, d)), rnd(seed + 3, (B, Hkv, L, d)),
            rnd(seed + 4, (B, L, Hq, d)), rnd(seed + 5, (B, Hkv, L, d)), rnd(seed + 6, (B, Hkv, L, d)))


def check(B, L, Hq, Hkv, d, bs, variant=0, seed=0):
    t = make(B, L, Hq, Hkv, d, seed)
    rOn, rLn, rOc, rLc = oracle.block_diffusion_train_attention(*t, bs=bs)
    On, Ln, Oc, Lc = gpu_train_attention(*t, bs=bs, variant=variant)
    assert attn_rel_err(On, rOn) <= TOL and attn_rel_err(Oc, rOc) <= TOL
    assert np.abs(Ln - rLn).max() <= LSE_TOL and np.abs(Lc - rLc).max() <= LSE_TOL


@pytest.mark.parametrize("variant", [0, 2, 3, 4, 5, 6, 7, 11])
def test_row_split_shapes(variant):
    check(B=2, L=204, Hq=4, Hkv=2, d=128, bs=4, variant=variant, seed=100)


@pytest.mark.parametrize("L,bs,Hq,Hkv,d", [(256, 32, 4, 4, 128), (130, 8, 6, 2, 64), (97, 1, 2, 2, 64),
                                           (64, 64, 2, 1, 128), (300, 16, 8, 2, 128)])
def test_block_sizes_and_heads(L, bs, Hq, Hkv, d):
    check(B=1, L=L, Hq=Hq, Hkv=Hkv, d=d, bs=bs, seed=200 + L)


def test_key_split_shape_with_rules():
    # a single query block (<= 32 rows per KV head) against long segments: the key-split kernel shape
    B, Lq, Hq, Hkv, d, bs, L = 2, 16, 2, 2, 128, 16, 400
    q = rnd(301, (B, Lq, Hq, d))
    kc, vc, kn, vn = rnd(302, (B, Hkv, L, d)), rnd(303, (B, Hkv, L, d)), rnd(304, (B, Hkv, L, d)), rnd(305, (B, Hkv, L, d))
    q_pos0 = 10 * bs
    ref, ref_lse = oracle.attention(q, [KV(kc, vc, 0, "earlier"), KV(kn, vn, 0, "same")], mask_mode="block_causal",
                                    bs=bs, q_pos0=q_pos0)
    out = torch.full((B, Lq, Hq, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    lse = torch.full((B, Hq, Lq), float("nan"), dtype=torch.float32, device=DEV)
    dlm.block_attn(bf16_dev(q), out, prefix=(bf16_dev(kc), bf16_dev(vc), 0, dlm.SEG_EARLIER_BLOCKS),
                   block=(bf16_dev(kn), bf16_dev(vn), 0, dlm.SEG_SAME_BLOCK), mask_mode=dlm.MASK_BLOCK_CAUSAL,
                   block_size=bs, q_pos0=q_pos0, lse=lse)
    torch.cuda.synchronize()
    assert attn_rel_err(bf16_host(out), ref) <= TOL
    assert np.abs(lse.cpu().numpy() - ref_lse).max() <= LSE_TOL


def test_first_block_sees_no_earlier_block():
    # rule EARLIER_BLOCKS alone: rows of block 0 see nothing -> zeros and lse = -inf, as the header states
    B, L, Hq, d, bs = 1, 40, 2, 64, 8
    q, k, v = rnd(401, (B, L, Hq, d)), rnd(402, (B, Hq, L, d)), rnd(403, (B, Hq, L, d))
    ref, ref_lse = oracle.attention(q, [KV(k, v, 0, "earlier")], mask_mode="block_causal", bs=bs)
    out = torch.full((B, L, Hq, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    lse = torch.full((B, Hq, L), float("nan"), dtype=torch.float32, device=DEV)
    dlm.block_attn(bf16_dev(q), out, block=(bf16_dev(k), bf16_dev(v), 0, dlm.SEG_EARLIER_BLOCKS),
                   mask_mode=dlm.MASK_BLOCK_CAUSAL, block_size=bs, lse=lse)
    torch.cuda.synchronize()
    got, got_lse = bf16_host(out), lse.cpu().numpy()
    assert not got[:, :bs].any() and np.all(np.isneginf(got_lse[:, :, :bs]))
    assert attn_rel_err(got[:, bs:], ref[:, bs:]) <= TOL
    assert np.abs(got_lse[:, :, bs:] - ref_lse[:, :, bs:]).max() <= LSE_TOL


def test_rules_are_refused_under_the_full_mask():
    z = torch.zeros((1, 8, 2, 64), dtype=torch.bfloat16, device=DEV)
    kv = torch.zeros((1, 2, 8, 64), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(dlm.DlmError):
        dlm.block_attn(z, z.clone(), block=(kv, kv, 0, dlm.SEG_SAME_BLOCK), mask_mode=dlm.MASK_FULL)


def test_full_size_training_pass_sampled_rows():
    """8 sequences of 4096 tokens, block size 4, 32 query / 8 KV heads of 128 (the full-sequence pass shape):
    sampled rows of both halves against the oracle."""
    cfg = synth.FULLPASS["c5b"].replace(B=8)
    qn, kn, vn = synth.fullpass_qkv(cfg)
    qc, kc, vc = synth.fullpass_qkv(cfg.replace(seed=cfg.seed + 1))
    print("inputs drawn", flush=True)
    On, Ln, Oc, Lc = gpu_train_attention(qn, kn, vn, qc, kc, vc, cfg.bs)
    rng = np.random.default_rng(1)
    n = 16
    rows = np.stack([rng.integers(0, cfg.B, n), rng.integers(0, cfg.Hq, n), rng.integers(0, cfg.L, n)], 1).astype(np.int32)
    rows[0], rows[1], rows[2] = (0, 0, 0), (cfg.B - 1, cfg.Hq - 1, cfg.L - 1), (1, 3, 5)
    rn, rln = oracle.attention(qn, [KV(kc, vc, 0, "earlier"), KV(kn, vn, 0, "same")], mask_mode="block_causal",
                               bs=cfg.bs, rows=rows)
    rc, rlc = oracle.attention(qc, [KV(kc, vc, 0)], mask_mode="block_causal", bs=cfg.bs, rows=rows)
    pick = lambda O: np.stack([O[b, i, h] for b, h, i in rows])
    assert attn_rel_err(pick(On), rn) <= TOL and attn_rel_err(pick(Oc), rc) <= TOL
    assert np.abs(np.array([Ln[b, h, i] for b, h, i in rows]) - rln).max() <= LSE_TOL
    assert np.abs(np.array([Lc[b, h, i] for b, h, i in rows]) - rlc).max() <= LSE_TOL
