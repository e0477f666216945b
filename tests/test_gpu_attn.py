"""dlm_block_attn against the oracle, element by element (GPU)."""
import numpy as np
import pytest
import torch

import oracle
from oracle import KV
from paper_2604_04215_amd import binding as dlm
from paper_2604_04215_amd import synth
from gpu_util import DEV, GuardedWorkspace, attn_rel_err, bf16_dev, bf16_host, dev, rnd

pytestmark = pytest.mark.gpu

TOL = 2e-2          # max relative error, bf16 operands with fp32 accumulation
LSE_TOL = 2e-3


def run_case(B, Lq, Hq, Hkv, d, P, Lb, S, mode="full", bs=0, q_pos0=None, plen=None, variant=0, seed=0,
             block_is_q=True, pos=None, split=None):
    """split: None = no workspace (the call cannot split the keys across workgroups); 0 = a workspace of the size the
    library asks for, split count chosen by the library; n >= 2 = that many splits asked for."""
    q = rnd(seed * 10 + 1, (B, Lq, Hq, d))
    Ltot = P + Lb + S
    k = rnd(seed * 10 + 2, (B, Hkv, Ltot, d))
    v = rnd(seed * 10 + 3, (B, Hkv, Ltot, d))
    q_pos0 = P if q_pos0 is None else q_pos0
    pos = (0, P, P + Lb) if pos is None else pos
    segs = [KV(k[:, :, :P], v[:, :, :P], pos[0]), KV(k[:, :, P:P + Lb], v[:, :, P:P + Lb], pos[1]),
            KV(k[:, :, P + Lb:], v[:, :, P + Lb:], pos[2])]
    ref, ref_lse = oracle.attention(q, segs, mask_mode=mode, bs=bs, q_pos0=q_pos0, prefix_len_b=plen)
    kd, vd, qd = bf16_dev(k), bf16_dev(v), bf16_dev(q)          # one cache tensor: segments are strided views
    out = torch.full((B, Lq, Hq, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    lse = torch.full((B, Hq, Lq), float("nan"), dtype=torch.float32, device=DEV)
    dlm.set_option("attn_variant", variant)
    gw = None
    try:
        kw = dict(prefix=(kd[:, :, :P], vd[:, :, :P], pos[0]) if P else None,
                  block=(kd[:, :, P:P + Lb], vd[:, :, P:P + Lb], pos[1]) if Lb else None,
                  suffix=(kd[:, :, P + Lb:], vd[:, :, P + Lb:], pos[2]) if S else None,
                  n_kv_heads=Hkv, mask_mode=dlm.MASK_BLOCK_CAUSAL if mode == "block_causal" else dlm.MASK_FULL,
                  block_size=bs, q_pos0=q_pos0,
                  prefix_len_b=None if plen is None else dev(np.asarray(plen, np.int32)))
        if split is not None:
            dlm.set_option("attn_split", split)
            need = dlm.block_attn_workspace_bytes(qd, **kw)
            assert need % (B * Hq * Lq * (d + 2) * 4) == 0 and need // (B * Hq * Lq * (d + 2) * 4) <= max(split, 16 * (split == 0))
            gw = GuardedWorkspace(need)          # exactly the size asked for, with guard bands
            kw["workspace"] = gw.ws if need else None
        dlm.block_attn(qd, out, lse=lse, **kw)
        torch.cuda.synchronize()
        if gw is not None:
            gw.check()
    finally:
        dlm.set_option("attn_variant", 0)
        dlm.set_option("attn_split", 0)
    err = attn_rel_err(bf16_host(out), ref)
    assert err <= TOL, f"attention rel err {err}"
    got_lse = lse.cpu().numpy().astype(np.float64)
    fin = np.isfinite(ref_lse)
    assert np.array_equal(np.isfinite(got_lse), fin)
    assert np.all(got_lse[~fin] == ref_lse[~fin])
    if fin.any():
        assert np.abs(got_lse[fin] - ref_lse[fin]).max() <= LSE_TOL
    return err


@pytest.mark.parametrize("variant", [0, 1, 2, 3, 8, 9, 10, 12, 13])
def test_rollout_shape_mha(variant):
    # block of 32 against a ragged prefix (several 32-key tiles and a tail), d = 128
    run_case(B=2, Lq=32, Hq=4, Hkv=4, d=128, P=200, Lb=32, S=0, variant=variant, seed=1)


@pytest.mark.parametrize("variant", [0, 2, 3, 4, 5, 6, 7, 11, 13, 14, 15])
def test_dual_cache_and_gqa7(variant):
    # 7 query heads per KV head (224 packed rows), prefix | block | suffix, ragged suffix
    run_case(B=2, Lq=32, Hq=14, Hkv=2, d=128, P=96, Lb=32, S=45, variant=variant, seed=2)


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("Lq,Hq,Hkv", [(1, 2, 2), (5, 4, 2), (32, 4, 4), (40, 6, 2), (70, 4, 1)])
def test_shapes(d, Lq, Hq, Hkv):
    run_case(B=2, Lq=Lq, Hq=Hq, Hkv=Hkv, d=d, P=77, Lb=Lq, S=9, seed=3 + Lq)


@pytest.mark.parametrize("variant", [0, 1, 2, 3, 4, 6, 12, 13, 14, 15])
@pytest.mark.parametrize("bs", [1, 4, 32])
def test_block_causal_rollout(variant, bs):
    # last block(s) of a block-diffusion sequence against the cache; positions are absolute
    run_case(B=2, Lq=8, Hq=8, Hkv=2, d=128, P=188, Lb=8, S=0, mode="block_causal", bs=bs, variant=variant, seed=5)


@pytest.mark.parametrize("variant", [0, 2, 3, 4, 6, 13, 14, 15])
def test_block_causal_full_sequence(variant):
    # training-style pass: Lq = Lk, bidirectional inside blocks of 4, causal across blocks
    B, L, Hq, Hkv, d = 2, 204, 4, 2, 128
    run_case(B=B, Lq=L, Hq=Hq, Hkv=Hkv, d=d, P=0, Lb=L, S=0, mode="block_causal", bs=4, q_pos0=0,
             variant=variant, seed=6)


def test_block_causal_hides_suffix_and_uses_positions():
    # suffix keys lie in later blocks: invisible; shifting every position by a block multiple changes nothing
    run_case(B=1, Lq=8, Hq=4, Hkv=2, d=64, P=40, Lb=8, S=16, mode="block_causal", bs=8, seed=7)
    run_case(B=1, Lq=8, Hq=4, Hkv=2, d=64, P=40, Lb=8, S=16, mode="block_causal", bs=8, q_pos0=1040,
             pos=(1000, 1040, 1048), seed=7)


def test_ragged_prefix_per_sequence():
    run_case(B=3, Lq=32, Hq=4, Hkv=2, d=128, P=100, Lb=32, S=20, plen=[100, 37, 0], seed=8)


@pytest.mark.parametrize("mode,bs", [("full", 0), ("block_causal", 4), ("block_causal", 32)])
@pytest.mark.parametrize("L", [1, 33, 64, 65, 97, 300])
def test_tile_counts_and_two_segments(mode, bs, L):
    # 1, 2, 3, 4 ... key tiles, even and odd counts, ragged tails; one segment and two (full-tile fast path of the
    # loads and stores next to the clamped path of the ragged last tile of each segment)
    run_case(B=1, Lq=L, Hq=4, Hkv=2, d=128, P=0, Lb=L, S=0, mode=mode, bs=bs, q_pos0=0, seed=40 + L)
    run_case(B=2, Lq=40, Hq=2, Hkv=2, d=128, P=L, Lb=40, S=0, mode=mode, bs=bs, seed=41 + L)


def test_degenerate_contexts():
    # no prefix and no suffix; a single key; no key at all (output 0, lse -inf)
    run_case(B=1, Lq=32, Hq=2, Hkv=2, d=128, P=0, Lb=32, S=0, seed=9)
    run_case(B=1, Lq=3, Hq=2, Hkv=1, d=64, P=1, Lb=0, S=0, seed=10)
    run_case(B=2, Lq=4, Hq=2, Hkv=2, d=128, P=5, Lb=0, S=0, plen=[0, 5], seed=11)


def test_noncontiguous_q_and_out_views():
    B, Lq, Hq, Hkv, d, P = 2, 32, 4, 4, 128, 64
    q = rnd(121, (B, Lq, Hq, d))
    k, v = rnd(122, (B, Hkv, P, d)), rnd(123, (B, Hkv, P, d))
    ref, _ = oracle.attention(q, [KV(k, v, 0)])
    big_q = torch.zeros((B, Lq, Hq + 2, d + 64), dtype=torch.bfloat16, device=DEV)
    big_o = torch.zeros_like(big_q)
    qv, ov = big_q[:, :, 1:1 + Hq, :d], big_o[:, :, 1:1 + Hq, :d]
    qv.copy_(bf16_dev(q))
    dlm.block_attn(qv, ov, prefix=(bf16_dev(k), bf16_dev(v), 0))
    torch.cuda.synchronize()
    assert attn_rel_err(bf16_host(ov), ref) <= TOL
    assert float(big_o[:, :, 0].abs().max()) == 0 and float(big_o[..., d:].abs().max()) == 0


def test_rerun_is_bitwise_identical():
    B, Lq, Hq, Hkv, d, P = 2, 32, 8, 2, 128, 300
    q, k, v = bf16_dev(rnd(131, (B, Lq, Hq, d))), bf16_dev(rnd(132, (B, Hkv, P, d))), bf16_dev(rnd(133, (B, Hkv, P, d)))
    o1, o2 = torch.empty_like(q), torch.empty_like(q)
    dlm.block_attn(q, o1, prefix=(k, v, 0))
    dlm.block_attn(q, o2, prefix=(k, v, 0))
    torch.cuda.synchronize()
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16))


@pytest.mark.parametrize("Lq,Hq,Hkv", [(8, 4, 4), (64, 8, 2)])
def test_peaked_softmax_large_scores(Lq, Hq, Hkv):
    """Scores of magnitude ~50 (Q and K four times the usual scale): nearly one-hot rows, the running maximum
    jumps by far more than the lazy-rescale threshold from tile to tile."""
    B, d, P = 2, 128, 300
    q = synth.f32_to_bf16_bits(np.random.default_rng(3).normal(size=(B, Lq, Hq, d)).astype(np.float32) * 4.0)
    k = synth.f32_to_bf16_bits(np.random.default_rng(4).normal(size=(B, Hkv, P, d)).astype(np.float32) * 4.0)
    v = rnd(305, (B, Hkv, P, d))
    ref, ref_lse = oracle.attention(q, [KV(k, v, 0)])
    out = torch.full((B, Lq, Hq, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    lse = torch.full((B, Hq, Lq), float("nan"), dtype=torch.float32, device=DEV)
    dlm.block_attn(bf16_dev(q), out, prefix=(bf16_dev(k), bf16_dev(v), 0), lse=lse)
    torch.cuda.synchronize()
    assert np.abs(ref_lse).max() > 50
    assert attn_rel_err(bf16_host(out), ref) <= TOL
    assert np.abs(lse.cpu().numpy() - ref_lse).max() <= 1e-4 * np.abs(ref_lse).max() + LSE_TOL


def test_non_temporal_kv_stream_changes_nothing():
    """g * Lq <= 32: one workgroup reads its K/V once, with non-temporal loads unless the option turns that off."""
    B, Lq, Hq, Hkv, d, P = 2, 8, 8, 2, 128, 500
    q, k, v = bf16_dev(rnd(141, (B, Lq, Hq, d))), bf16_dev(rnd(142, (B, Hkv, P, d))), bf16_dev(rnd(143, (B, Hkv, P, d)))
    o1, o2 = torch.empty_like(q), torch.empty_like(q)
    dlm.block_attn(q, o1, prefix=(k, v, 0))
    dlm.set_option("attn_nt", 0)
    try:
        dlm.block_attn(q, o2, prefix=(k, v, 0))
    finally:
        dlm.set_option("attn_nt", 1)
    torch.cuda.synchronize()
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16))
    ref, _ = oracle.attention(rnd(141, (B, Lq, Hq, d)), [KV(rnd(142, (B, Hkv, P, d)), rnd(143, (B, Hkv, P, d)), 0)])
    assert attn_rel_err(bf16_host(o1), ref) <= TOL


@pytest.mark.parametrize("B,Hkv,g,Lq", [(1, 1, 2, 300), (1, 3, 4, 130), (2, 2, 1, 700), (4, 2, 2, 129), (3, 4, 2, 257)])
@pytest.mark.parametrize("variant", [4, 6, 11, 13, 15])
def test_xcd_grouped_grid_covers_every_tile_once(B, Hkv, g, Lq, variant):
    """Group counts 1, 3, 4, 8, 12 (tiles of a group dealt to 8, 8, 2, 1, 2 XCDs) and ragged tile counts, both masks:
    the 1-D grid must produce what the plain (tile, KV head, sequence) grid does, bit for bit, and the oracle's result."""
    d, P = 64, 40
    for mode, bs in (("full", 0), ("block_causal", 8)):
        run_case(B=B, Lq=Lq, Hq=Hkv * g, Hkv=Hkv, d=d, P=P, Lb=Lq, S=0, mode=mode, bs=bs, variant=variant, seed=900 + Lq)
        q = bf16_dev(rnd(9001, (B, Lq, Hkv * g, d)))
        k, v = bf16_dev(rnd(9002, (B, Hkv, Lq, d))), bf16_dev(rnd(9003, (B, Hkv, Lq, d)))
        outs = []
        dlm.set_option("attn_variant", variant)
        try:
            for remap in (7, 1, 0):
                dlm.set_option("attn_remap", remap)
                o = torch.full_like(q, float("nan"))
                dlm.block_attn(q, o, block=(k, v, 0), mask_mode=dlm.MASK_BLOCK_CAUSAL if bs else dlm.MASK_FULL, block_size=bs)
                torch.cuda.synchronize()
                outs.append(o.view(torch.int16))
        finally:
            dlm.set_option("attn_remap", 7)
            dlm.set_option("attn_variant", 0)
        assert torch.equal(outs[0], outs[2]) and torch.equal(outs[1], outs[2])


@pytest.mark.parametrize("Lq,Hq,Hkv,variant", [(32, 4, 4, 0), (8, 8, 2, 0), (130, 4, 2, 0), (130, 4, 2, 11), (300, 2, 1, 6)])
def test_sequences_flagged_inactive_are_skipped(Lq, Hq, Hkv, variant):
    """seq_active[b] == 0: the sequence's rows of out and lse keep what they held; the others match the oracle."""
    B, d, P = 5, 64, 70
    q, k, v = rnd(151, (B, Lq, Hq, d)), rnd(152, (B, Hkv, P + Lq, d)), rnd(153, (B, Hkv, P + Lq, d))
    ref, ref_lse = oracle.attention(q, [KV(k[:, :, :P], v[:, :, :P], 0), KV(k[:, :, P:], v[:, :, P:], P)])
    kd, vd = bf16_dev(k), bf16_dev(v)
    active = np.array([3, 0, 1, 0, -2], np.int32)          # any non-zero value counts as active
    out = torch.full((B, Lq, Hq, d), 7.0, dtype=torch.bfloat16, device=DEV)
    lse = torch.full((B, Hq, Lq), -3.0, dtype=torch.float32, device=DEV)
    dlm.set_option("attn_variant", variant)
    try:
        dlm.block_attn(bf16_dev(q), out, prefix=(kd[:, :, :P], vd[:, :, :P], 0), block=(kd[:, :, P:], vd[:, :, P:], P),
                       lse=lse, seq_active=dev(active))
        torch.cuda.synchronize()
    finally:
        dlm.set_option("attn_variant", 0)
    on = active != 0
    assert attn_rel_err(bf16_host(out)[on], ref[on]) <= TOL
    assert np.abs(lse.cpu().numpy()[on] - ref_lse[on]).max() <= LSE_TOL
    assert bool((out[~torch.from_numpy(on).to(DEV)] == 7.0).all()) and bool((lse[~torch.from_numpy(on).to(DEV)] == -3.0).all())


@pytest.mark.parametrize("variant", [0, 1, 2, 12, 13, 14, 15])
def test_planted_one_hot_values_expose_every_key(variant):
    """V[j] = e_(j mod d): output channel c is the total probability of keys j = c (mod d), so a
    dropped, duplicated or misplaced key shifts some channel by a large relative amount; with Q = 0
    every probability is exactly 1/Lk."""
    B, Lq, Hq, Hkv, d, P, Lb, S = 1, 32, 2, 2, 64, 150, 32, 21
    Lk = P + Lb + S
    v = np.zeros((B, Hkv, Lk, d), np.float32)
    v[:, :, np.arange(Lk), np.arange(Lk) % d] = 1.0
    from paper_2604_04215_amd import synth
    vb = synth.f32_to_bf16_bits(v)
    k = rnd(201, (B, Hkv, Lk, d))
    for qbits in (np.zeros((B, Lq, Hq, d), np.uint16), rnd(202, (B, Lq, Hq, d), 0.3)):
        segs = [KV(k[:, :, :P], vb[:, :, :P], 0), KV(k[:, :, P:P + Lb], vb[:, :, P:P + Lb], P),
                KV(k[:, :, P + Lb:], vb[:, :, P + Lb:], P + Lb)]
        ref, _ = oracle.attention(qbits, segs)
        kd, vd = bf16_dev(k), bf16_dev(vb)
        out = torch.empty((B, Lq, Hq, d), dtype=torch.bfloat16, device=DEV)
        dlm.set_option("attn_variant", variant)
        try:
            dlm.block_attn(bf16_dev(qbits), out, prefix=(kd[:, :, :P], vd[:, :, :P], 0),
                           block=(kd[:, :, P:P + Lb], vd[:, :, P:P + Lb], P),
                           suffix=(kd[:, :, P + Lb:], vd[:, :, P + Lb:], P + Lb))
            torch.cuda.synchronize()
        finally:
            dlm.set_option("attn_variant", 0)
        from paper_2604_04215_amd.synth import bf16_bits_to_f64
        got = bf16_bits_to_f64(bf16_host(out))
        # every channel is a sum of 3-4 probabilities: a per-element relative check is meaningful here
        assert np.abs(got - ref).max() <= 2e-2 * ref.min()


def test_prefix_only_cache_with_block_and_suffix_queries():
    """Prefix-only caching: only the prompt and finished blocks are cached, and the step recomputes the current
    block AND the still-masked suffix, so the query set is block + suffix (Lq = Lb + S) against
    [cached prefix | those same Lb + S fresh rows].  Same kernel, larger Lq."""
    for Lb, S, P in [(32, 96, 200), (32, 224, 72)]:
        run_case(B=2, Lq=Lb + S, Hq=4, Hkv=2, d=128, P=P, Lb=Lb + S, S=0, seed=77 + S)


def test_largest_batch_the_grid_takes():
    """B = 65535 (the launch grid's limit; one more is refused): one query row, one key, per sequence."""
    B, d = 65535, 64
    q, k, v = rnd(991, (B, 1, 1, d)), rnd(992, (B, 1, 1, d)), rnd(993, (B, 1, 1, d))
    out = torch.full((B, 1, 1, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    dlm.block_attn(bf16_dev(q), out, block=(bf16_dev(k), bf16_dev(v), 0))
    torch.cuda.synchronize()
    got = synth.bf16_bits_to_f64(bf16_host(out)).reshape(B, d)
    assert np.array_equal(got, synth.bf16_bits_to_f64(v).reshape(B, d))        # softmax over one key: O = V exactly
    big = torch.zeros((65536, 1, 1, d), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(dlm.DlmError):
        dlm.block_attn(big, big.clone(), block=(big.view(65536, 1, 1, d), big.view(65536, 1, 1, d), 0))


# ---- key split across workgroups + merge kernel ------------------------------------------------------------
@pytest.mark.parametrize("variant", [0, 1, 12, 8])
@pytest.mark.parametrize("split", [2, 3, 5])
def test_key_split_rollout_shape(variant, split):
    """One workgroup per (sequence, KV head) split into `split` workgroups over the key tiles: ragged prefix (a tail
    tile), block and suffix segments, d = 128 and 64; every element against the oracle."""
    run_case(B=2, Lq=32, Hq=4, Hkv=4, d=128, P=712, Lb=32, S=100, variant=variant, seed=41, split=split)
    run_case(B=3, Lq=16, Hq=4, Hkv=2, d=64, P=1000, Lb=16, S=0, variant=variant, seed=42, split=split)


@pytest.mark.parametrize("variant", [0, 2, 3, 4, 6, 11, 13, 14, 15])
@pytest.mark.parametrize("split", [2, 3])
def test_key_split_row_tile_shapes(variant, split):
    """128- / 256-row workgroups (7 heads per KV head x 32 rows = 224 rows, two ragged row tiles) with the keys split
    across workgroups, full and block-causal masks, plain and XCD-grouped grids."""
    run_case(B=2, Lq=32, Hq=14, Hkv=2, d=128, P=640, Lb=32, S=0, variant=variant, seed=43, split=split)
    run_case(B=1, Lq=160, Hq=4, Hkv=2, d=128, P=96, Lb=160, S=0, mode="block_causal", bs=32, q_pos0=96, variant=variant,
             seed=44, split=split)
    dlm.set_option("attn_remap", 0)
    try:
        run_case(B=2, Lq=40, Hq=8, Hkv=2, d=64, P=520, Lb=40, S=30, variant=variant, seed=45, split=split)
    finally:
        dlm.set_option("attn_remap", 7)


def test_key_split_edge_cases():
    """More splits than a sequence has key tiles (some workgroups get none), sequences whose prefix is empty, rows
    that see no key at all, and a split count the library lowers because the problem has few tiles."""
    # ragged per-sequence prefix: sequence 1 has no prefix at all, sequence 2 a single key
    run_case(B=3, Lq=32, Hq=2, Hkv=2, d=128, P=640, Lb=32, S=0, plen=[640, 0, 1], variant=1, seed=46, split=5)
    run_case(B=3, Lq=32, Hq=2, Hkv=2, d=128, P=640, Lb=32, S=0, plen=[640, 0, 1], variant=4, seed=46, split=4)
    # block-causal where early rows see only the first keys: splits past their visible range hold nothing for them
    run_case(B=1, Lq=64, Hq=2, Hkv=1, d=128, P=0, Lb=640, S=0, mode="block_causal", bs=4, q_pos0=0, variant=1, seed=47, split=4)
    run_case(B=1, Lq=256, Hq=2, Hkv=1, d=128, P=0, Lb=640, S=0, mode="block_causal", bs=4, q_pos0=0, variant=6, seed=47, split=4)
    # few tiles: the library lowers the split count (at least four tiles per workgroup) or drops the split
    run_case(B=1, Lq=32, Hq=2, Hkv=2, d=64, P=100, Lb=32, S=0, variant=0, seed=48, split=6)
    # library-chosen split: 16 workgroups unsplit and 64 key tiles -> 16 splits of 4 tiles; 8 of 128 rows -> 16 splits
    run_case(B=2, Lq=32, Hq=8, Hkv=8, d=128, P=2016, Lb=32, S=0, variant=0, seed=49, split=0)
    run_case(B=1, Lq=32, Hq=32, Hkv=8, d=128, P=2080, Lb=32, S=0, variant=0, seed=50, split=0)
    q = torch.zeros((2, 32, 8, 128), dtype=torch.bfloat16, device=DEV)
    k = torch.zeros((2, 8, 2048, 128), dtype=torch.bfloat16, device=DEV)
    assert dlm.block_attn_workspace_bytes(q, block=(k, k, 0)) == 16 * 2 * 8 * 32 * 130 * 4
    assert dlm.block_attn_workspace_bytes(q, block=(k[:, :, :992], k[:, :, :992], 0)) == 0      # 31 tiles: too few to pay


def test_key_split_is_deterministic_and_skips_inactive_sequences():
    B, Lq, H, d, P = 4, 32, 4, 128, 800
    q = bf16_dev(rnd(5001, (B, Lq, H, d)))
    k, v = bf16_dev(rnd(5002, (B, H, P + Lq, d))), bf16_dev(rnd(5003, (B, H, P + Lq, d)))
    kw = dict(prefix=(k[:, :, :P], v[:, :, :P], 0), block=(k[:, :, P:], v[:, :, P:], P))
    dlm.set_option("attn_split", 3)
    try:
        ws = torch.empty(dlm.block_attn_workspace_bytes(q, **kw), dtype=torch.uint8, device=DEV)
        assert ws.numel() == 3 * B * H * Lq * (d + 2) * 4
        outs = []
        for _ in range(2):
            ws.fill_(0xFF)                                   # whatever the workspace held before must not matter
            o = torch.full_like(q, float("nan"))
            lse = torch.full((B, H, Lq), float("nan"), device=DEV)
            dlm.block_attn(q, o, lse=lse, workspace=ws, **kw)
            torch.cuda.synchronize()
            outs.append((o.view(torch.int16).clone(), lse.clone()))
        assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
        # unsplit result: same values up to the rounding of a different summation order
        dlm.set_option("attn_split", 1)
        o1 = torch.full_like(q, float("nan"))
        dlm.block_attn(q, o1, workspace=ws, **kw)
        torch.cuda.synchronize()
        assert (outs[0][0].view(torch.bfloat16).float() - o1.float()).abs().max().item() <= 2e-2
        # sequences 1 and 3 inactive: their rows keep the sentinel, the others equal the full run
        dlm.set_option("attn_split", 3)
        act = dev(np.array([1, 0, 5, 0], np.int32))
        o2 = torch.full_like(q, 7.0)
        dlm.block_attn(q, o2, workspace=ws, seq_active=act, **kw)
        torch.cuda.synchronize()
        assert torch.equal(o2.view(torch.int16)[[0, 2]], outs[0][0][[0, 2]])
        assert (o2[[1, 3]] == 7.0).all().item()
        # a workspace that is too small: the call runs unsplit instead of failing
        o3 = torch.full_like(q, float("nan"))
        dlm.block_attn(q, o3, workspace=ws[:1024], **kw)
        torch.cuda.synchronize()
        assert torch.equal(o3.view(torch.int16), o1.view(torch.int16))
    finally:
        dlm.set_option("attn_split", 0)


@pytest.mark.parametrize("variant", [13, 14, 15])
def test_two_key_groups_per_workgroup_edge_cases(variant):
    """128-row workgroups whose eight wavefronts form two key groups: odd tile counts (the second group's last tile
    does not exist), a single tile, ragged per-sequence prefixes down to none, d = 64, rows that see nothing."""
    run_case(B=3, Lq=32, Hq=4, Hkv=2, d=128, P=100, Lb=32, S=20, plen=[100, 37, 0], variant=variant, seed=61)
    run_case(B=1, Lq=130, Hq=2, Hkv=1, d=64, P=0, Lb=20, S=0, variant=variant, seed=62)            # one tile only
    run_case(B=2, Lq=70, Hq=6, Hkv=2, d=64, P=333, Lb=70, S=11, variant=variant, seed=63)
    run_case(B=1, Lq=200, Hq=2, Hkv=1, d=128, P=0, Lb=200, S=0, mode="block_causal", bs=4, q_pos0=0, variant=variant, seed=64)
    run_case(B=2, Lq=4, Hq=2, Hkv=2, d=128, P=5, Lb=0, S=0, plen=[0, 5], variant=variant, seed=65)
