"""dlm_block_attn_bwd against the oracle's gradients (GPU).

The forward results the gradient kernels consume (O and LSE) come from dlm_block_attn itself, as in training.
Two bounds per gradient tensor:
  * element-wise, the forward pass's metric |got - ref| / max(|ref|, rms of the reference row over head_dim),
    at 4e-2: besides the bf16 rounding of dS (2^-9) and of the result, delta = rowsum(dO * O) is formed from the
    bf16 forward output, and for a row that sees only a few keys that error (about sqrt(d) * 2^-9 * |O|) shifts
    every dS of the row the same way; a float64 emulation of exactly these roundings gives 2.3e-2 on the worst
    case here (block size 7, first block), of which 1.4e-2 is the delta term;
  * in aggregate, ||got - ref||_F / ||ref||_F <= 1e-2 (the same emulation: 2.5e-3): a wrong scale, a missing
    term or a misplaced mask shows up here long before it reaches the element-wise bound."""
import numpy as np
import pytest
import torch

from oracle import KV
from oracle import backward as obw
from paper_2604_04215_amd import binding as dlm
from paper_2604_04215_amd import synth
from gpu_util import DEV, GuardedWorkspace, attn_rel_err, bf16_dev, bf16_host, dev, rnd

pytestmark = pytest.mark.gpu

TOL = 4e-2
FRO_TOL = 1e-2


def fro_err(got_u16, ref):
    got = synth.bf16_bits_to_f64(got_u16).reshape(ref.shape)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.abs(got).max())
RULES = {"causal": dlm.SEG_CAUSAL, "earlier": dlm.SEG_EARLIER_BLOCKS, "same": dlm.SEG_SAME_BLOCK}


def run_bwd(q, segs, d_out, mode="full", bs=0, q_pos0=0, want=(True, True, True)):
    """segs: list of up to 3 oracle KV (prefix, block, suffix order; None for absent)."""
    B, Lq, Hq, d = q.shape
    qd, dod = bf16_dev(q), bf16_dev(d_out)
    out = torch.empty((B, Lq, Hq, d), dtype=torch.bfloat16, device=DEV)
    lse = torch.empty((B, Hq, Lq), dtype=torch.float32, device=DEV)
    tup, grads = [], []
    for s in segs:
        if s is None:
            tup.append(None)
            grads.append(None)
            continue
        kd, vd = bf16_dev(s.k), bf16_dev(s.v)
        tup.append((kd, vd, s.pos0, RULES[s.rule]))
        grads.append((torch.full_like(kd, float("nan")), torch.full_like(vd, float("nan"))))
    mm = dlm.MASK_BLOCK_CAUSAL if mode == "block_causal" else dlm.MASK_FULL
    dlm.block_attn(qd, out, prefix=tup[0], block=tup[1], suffix=tup[2], mask_mode=mm, block_size=bs, q_pos0=q_pos0, lse=lse)
    dq = torch.full_like(qd, float("nan"))
    gw = GuardedWorkspace(dlm.block_attn_bwd_workspace_bytes(B * Lq, Hq))   # exactly the size asked for, guarded
    dlm.block_attn_bwd(qd, out, dod, lse, dq, prefix=tup[0], block=tup[1], suffix=tup[2],
                       d_prefix=grads[0], d_block=grads[1], d_suffix=grads[2],
                       mask_mode=mm, block_size=bs, q_pos0=q_pos0, workspace=gw.ws)
    gw.check()
    return bf16_host(dq), [None if g is None else (bf16_host(g[0]), bf16_host(g[1])) for g in grads]


def check(q, segs, d_out, **kw):
    dq, grads = run_bwd(q, segs, d_out, **kw)
    present = [s for s in segs if s is not None]
    rdq, rg = obw.attention_backward(q, present, d_out, mask_mode=kw.get("mode", "full"), bs=kw.get("bs", 0),
                                     q_pos0=kw.get("q_pos0", 0))
    errs, fro = [attn_rel_err(dq, rdq)], [fro_err(dq, rdq)]
    for g, (rk, rv) in zip([g for g in grads if g is not None], rg):
        errs += [attn_rel_err(g[0], rk), attn_rel_err(g[1], rv)]
        fro += [fro_err(g[0], rk), fro_err(g[1], rv)]
    assert max(errs) <= TOL, f"gradient rel errs {errs}"
    assert max(fro) <= FRO_TOL, f"gradient Frobenius errs {fro}"
    return errs


def make(B, Lq, Hq, Hkv, d, lens, seed, pos=None, rules=None):
    q, d_out = rnd(seed + 1, (B, Lq, Hq, d)), rnd(seed + 2, (B, Lq, Hq, d))
    segs, p0 = [], 0
    for n, L in enumerate(lens):
        if L == 0:
            segs.append(None)
            continue
        segs.append(KV(rnd(seed + 10 + n, (B, Hkv, L, d)), rnd(seed + 20 + n, (B, Hkv, L, d)),
                       p0 if pos is None else pos[n], "causal" if rules is None else rules[n]))
        p0 += L
    return q, segs, d_out


@pytest.mark.parametrize("Lq,Hq,Hkv,d,L", [(64, 4, 4, 128, 64), (100, 4, 2, 128, 100), (33, 6, 2, 64, 33),
                                          (200, 2, 1, 64, 200), (1, 2, 2, 128, 1), (129, 8, 2, 128, 129)])
def test_full_mask_self_attention(Lq, Hq, Hkv, d, L):
    q, segs, d_out = make(2, Lq, Hq, Hkv, d, (0, L, 0), seed=Lq)
    check(q, segs, d_out)


def test_three_segments_full_mask():
    q, segs, d_out = make(2, 40, 4, 2, 128, (70, 40, 50), seed=500)
    check(q, segs, d_out)


@pytest.mark.parametrize("bs", [4, 32, 7])
def test_block_causal_self_attention(bs):
    q, segs, d_out = make(2, 150, 4, 2, 128, (0, 150, 0), seed=600 + bs)
    check(q, segs, d_out, mode="block_causal", bs=bs)


def test_block_causal_with_prefix_and_offset():
    q, segs, d_out = make(1, 48, 4, 4, 64, (80, 48, 32), seed=700)
    check(q, segs, d_out, mode="block_causal", bs=16, q_pos0=80)


@pytest.mark.parametrize("L,bs", [(204, 4), (128, 32), (70, 8)])
def test_block_diffusion_training_mask(L, bs):
    # noisy half: prefix = clean K/V (earlier blocks), block = noisy K/V (own block), both at position 0
    q, segs, d_out = make(2, L, 4, 2, 128, (L, L, 0), seed=800 + L, pos=(0, 0, 0), rules=("earlier", "same", "causal"))
    check(q, segs, d_out, mode="block_causal", bs=bs)


def test_gradients_not_wanted_are_skipped():
    q, segs, d_out = make(1, 64, 2, 2, 64, (32, 64, 0), seed=900)
    B, Lq, Hq, d = q.shape
    qd, dod = bf16_dev(q), bf16_dev(d_out)
    out = torch.empty((B, Lq, Hq, d), dtype=torch.bfloat16, device=DEV)
    lse = torch.empty((B, Hq, Lq), dtype=torch.float32, device=DEV)
    pk, pv, bk, bv = bf16_dev(segs[0].k), bf16_dev(segs[0].v), bf16_dev(segs[1].k), bf16_dev(segs[1].v)
    dlm.block_attn(qd, out, prefix=(pk, pv, 0), block=(bk, bv, 32), lse=lse)
    dbk, dbv = torch.zeros_like(bk), torch.zeros_like(bv)
    ws = torch.empty(dlm.block_attn_bwd_workspace_bytes(B * Lq, Hq), dtype=torch.uint8, device=DEV)
    dlm.block_attn_bwd(qd, out, dod, lse, None, prefix=(pk, pv, 0), block=(bk, bv, 32), d_block=(dbk, dbv), workspace=ws)
    torch.cuda.synchronize()
    _, rg = obw.attention_backward(q, segs[:2], d_out)
    assert attn_rel_err(bf16_host(dbk), rg[1][0]) <= TOL and attn_rel_err(bf16_host(dbv), rg[1][1]) <= TOL
    assert fro_err(bf16_host(dbk), rg[1][0]) <= FRO_TOL and fro_err(bf16_host(dbv), rg[1][1]) <= FRO_TOL
    with pytest.raises(dlm.DlmError):
        dlm.block_attn_bwd(qd, out, dod, lse, None, block=(bk, bv, 32), d_block=(dbk, dbv), workspace=ws[:16])


def test_packed_variable_length():
    lens = np.array([70, 1, 0, 130, 33], np.int64)
    T, Hq, Hkv, d = int(lens.sum()), 4, 2, 128
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    q, k, v, d_out = rnd(31, (T, Hq, d)), rnd(32, (T, Hkv, d)), rnd(33, (T, Hkv, d)), rnd(34, (T, Hq, d))
    qd, kd, vd, dod = bf16_dev(q), bf16_dev(k), bf16_dev(v), bf16_dev(d_out)
    out = torch.empty_like(qd)
    lse = torch.empty((Hq, T), dtype=torch.float32, device=DEV)
    mx = int(lens.max())
    dlm.varlen_attn(qd, kd, vd, out, dev(cu), mx, lse=lse)
    dq, dk, dv = (torch.full_like(t, float("nan")) for t in (qd, kd, vd))
    ws = torch.empty(dlm.block_attn_bwd_workspace_bytes(T, Hq), dtype=torch.uint8, device=DEV)
    dlm.block_attn_bwd(qd, out, dod, lse, dq, block=(kd, vd), d_block=(dk, dv), cu_seqlens=dev(cu), max_seqlen=mx, workspace=ws)
    torch.cuda.synchronize()
    gq, gk, gv = bf16_host(dq), bf16_host(dk), bf16_host(dv)
    for b in range(len(lens)):
        a, e = cu[b], cu[b + 1]
        if e == a:
            continue
        seg = KV(np.ascontiguousarray(k[a:e].transpose(1, 0, 2))[None], np.ascontiguousarray(v[a:e].transpose(1, 0, 2))[None], 0)
        rq, [(rk, rv)] = obw.attention_backward(q[a:e][None], [seg], d_out[a:e][None])
        assert attn_rel_err(gq[a:e], rq[0]) <= TOL
        assert attn_rel_err(gk[a:e], rk[0].transpose(1, 0, 2)) <= TOL
        assert attn_rel_err(gv[a:e], rv[0].transpose(1, 0, 2)) <= TOL
        assert max(fro_err(gq[a:e], rq[0]), fro_err(gk[a:e], rk[0].transpose(1, 0, 2)),
                   fro_err(gv[a:e], rv[0].transpose(1, 0, 2))) <= FRO_TOL


def test_full_size_training_shape_sampled_against_oracle():
    """2 sequences of 4096 tokens, block size 4, 32 query / 8 KV heads of 128, block-causal: gradients of one
    (sequence, KV head) slice against the oracle (the dense float64 oracle handles 4096 x 4096 per head)."""
    cfg = synth.FULLPASS["c5b"].replace(B=2)
    q, k, v = synth.fullpass_qkv(cfg)
    d_out = rnd(4242, q.shape)
    B, L, Hq, d = q.shape
    qd, kd, vd, dod = bf16_dev(q), bf16_dev(k), bf16_dev(v), bf16_dev(d_out)
    out = torch.empty_like(qd)
    lse = torch.empty((B, Hq, L), dtype=torch.float32, device=DEV)
    dlm.block_attn(qd, out, block=(kd, vd, 0), mask_mode=dlm.MASK_BLOCK_CAUSAL, block_size=cfg.bs, lse=lse)
    dq, dk, dv = torch.empty_like(qd), torch.empty_like(kd), torch.empty_like(vd)
    ws = torch.empty(dlm.block_attn_bwd_workspace_bytes(B * L, Hq), dtype=torch.uint8, device=DEV)
    dlm.block_attn_bwd(qd, out, dod, lse, dq, block=(kd, vd, 0), d_block=(dk, dv), mask_mode=dlm.MASK_BLOCK_CAUSAL,
                       block_size=cfg.bs, workspace=ws)
    torch.cuda.synchronize()
    print("gpu done", flush=True)
    b, kvh, g = 1, 5, cfg.Hq // cfg.Hkv
    hs = slice(kvh * g, (kvh + 1) * g)
    rq, [(rk, rv)] = obw.attention_backward(q[b:b + 1, :, hs], [KV(k[b:b + 1, kvh:kvh + 1], v[b:b + 1, kvh:kvh + 1], 0)],
                                            d_out[b:b + 1, :, hs], mask_mode="block_causal", bs=cfg.bs)
    gq, gk, gv = bf16_host(dq)[b:b + 1, :, hs], bf16_host(dk)[b:b + 1, kvh:kvh + 1], bf16_host(dv)[b:b + 1, kvh:kvh + 1]
    assert max(attn_rel_err(gq, rq), attn_rel_err(gk, rk), attn_rel_err(gv, rv)) <= TOL
    assert max(fro_err(gq, rq), fro_err(gk, rk), fro_err(gv, rv)) <= FRO_TOL


@pytest.mark.parametrize("B,Hkv,g,L", [(1, 1, 2, 600), (1, 3, 4, 300), (4, 2, 2, 520)])
def test_xcd_grouped_grids_give_the_plain_grids_bits(B, Hkv, g, L):
    """Group counts 1, 3, 8: the 1-D grids of the dQ and dK / dV passes against the plain ones, bit for bit, and the
    oracle's gradients; 520 and 600 keys make 5 slabs, so block-causal slabs are paired (second one walked upwards)."""
    for mode, bs in (("full", 0), ("block_causal", 8)):
        q, segs, d_out = make(B, L, Hkv * g, Hkv, 64, (0, L, 0), seed=1200 + L)
        res = []
        try:
            for remap in (7, 0):
                dlm.set_option("attn_remap", remap)
                res.append(run_bwd(q, segs, d_out, mode=mode, bs=bs))
        finally:
            dlm.set_option("attn_remap", 7)
        assert np.array_equal(res[0][0], res[1][0])
        assert np.array_equal(res[0][1][1][0], res[1][1][1][0]) and np.array_equal(res[0][1][1][1], res[1][1][1][1])
        check(q, segs, d_out, mode=mode, bs=bs)
