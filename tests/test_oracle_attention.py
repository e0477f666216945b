"""Pins for the oracle's attention (CPU only): brute force, closed forms, metamorphic
identities, textbook special cases.  Each is chosen so that a plausible slip in the
oracle (dropped scale, wrong GQA map, transposed operand, off-by-one block rule,
ignored segment, mishandled ragged prefix) fails at least one of them."""
import math

import numpy as np
import pytest

import oracle
from oracle import KV
from paper_2604_04215_amd import synth
from brute_force import attention_brute, bf16_to_float


def rnd(seed, shape, std=1.0):
    return synth.normal_bf16(1234, 77, (seed,), shape, std)


def to_lists(u16):
    return synth.bf16_bits_to_f64(u16).tolist()


def f64(u16):
    return synth.bf16_bits_to_f64(u16)


@pytest.mark.parametrize("mode,bs", [("full", 0), ("block_causal", 4), ("block_causal", 3)])
def test_brute_force_tiny(mode, bs):
    B, Lq, Hq, Hkv, d = 2, 5, 4, 2, 8
    P, S = 7, 3
    q = rnd(1, (B, Lq, Hq, d))
    kp, vp = rnd(2, (B, Hkv, P, d)), rnd(3, (B, Hkv, P, d))
    kb, vb = rnd(4, (B, Hkv, Lq, d)), rnd(5, (B, Hkv, Lq, d))
    ks, vs = rnd(6, (B, Hkv, S, d)), rnd(7, (B, Hkv, S, d))
    plen = np.array([7, 4], dtype=np.int32)
    O, lse = oracle.attention(q, [KV(kp, vp, 0), KV(kb, vb, P), KV(ks, vs, P + Lq)],
                              mask_mode=mode, bs=bs, q_pos0=P, prefix_len_b=plen)
    kcat = np.concatenate([kp, kb, ks], axis=2)
    vcat = np.concatenate([vp, vb, vs], axis=2)
    key_ok = [[1 if (j >= P or j < plen[b]) else 0 for j in range(P + Lq + S)] for b in range(B)]
    Ob, lb = attention_brute(to_lists(q), to_lists(kcat), to_lists(vcat), list(range(P + Lq + S)),
                             P, mode, bs, key_ok=key_ok)
    assert np.allclose(O, np.array(Ob), rtol=0, atol=1e-12)
    assert np.allclose(lse, np.array(lb), rtol=0, atol=1e-12)
    if mode == "block_causal":
        # the rule really hides something: suffix keys (later blocks) must not matter
        O2, _ = oracle.attention(q, [KV(kp, vp, 0), KV(kb, vb, P)], mask_mode=mode, bs=bs, q_pos0=P,
                                 prefix_len_b=plen)
        assert (P + Lq) % bs == 0
        assert np.array_equal(O, O2)


def test_closed_forms():
    B, Lq, H, d, Lk = 1, 3, 2, 16, 11
    q = rnd(10, (B, Lq, H, d))
    v = rnd(11, (B, H, Lk, d))
    # identical keys -> uniform weights -> mean of V rows
    k_same = np.repeat(rnd(12, (B, H, 1, d)), Lk, axis=2)
    O, lse = oracle.attention(q, [KV(k_same, v, 0)])
    want = f64(v).mean(axis=2)                       # [B,H,d]
    for i in range(Lq):
        assert np.allclose(O[:, i], want, atol=1e-13)
    # lse = s + log(Lk) with s = scale * q.k
    s = np.einsum("bihd,bhd->bhi", f64(q), f64(k_same)[:, :, 0]) / math.sqrt(d)
    assert np.allclose(lse, s + math.log(Lk), atol=1e-12)
    # Q = 0 -> uniform mean as well, lse = log(Lk)
    k = rnd(13, (B, H, Lk, d))
    O0, lse0 = oracle.attention(np.zeros_like(q), [KV(k, v, 0)])
    for i in range(Lq):
        assert np.allclose(O0[:, i], want, atol=1e-13)
    assert np.allclose(lse0, math.log(Lk), atol=1e-13)
    # constant V -> that constant
    vconst = np.repeat(rnd(14, (B, H, 1, d)), Lk, axis=2)
    Oc, _ = oracle.attention(q, [KV(k, vconst, 0)])
    for i in range(Lq):
        assert np.allclose(Oc[:, i], f64(vconst)[:, :, 0], atol=1e-13)


def test_dominant_key_selects_its_value_row():
    # one key aligned with q with a huge score: softmax -> one-hot (gap >= 40 in the exponent)
    d, Lk = 16, 9
    qv = np.zeros((1, 1, 1, d), np.float32)
    qv[..., 0] = 64.0
    kf = np.zeros((1, 1, Lk, d), np.float32)
    kf[0, 0, 4, 0] = 8.0                                   # score = 64*8/4 = 128, others 0
    v = rnd(15, (1, 1, Lk, d))
    O, lse = oracle.attention(synth.f32_to_bf16_bits(qv), [KV(synth.f32_to_bf16_bits(kf), v, 0)])
    assert np.allclose(O[0, 0, 0], f64(v)[0, 0, 4], atol=1e-15)
    assert abs(lse[0, 0, 0] - 128.0) < 1e-12


def test_scale_argument_and_default():
    q, k, v = rnd(20, (1, 2, 1, 8)), rnd(21, (1, 1, 5, 8)), rnd(22, (1, 1, 5, 8))
    O1, l1 = oracle.attention(q, [KV(k, v, 0)])
    O2, l2 = oracle.attention(q, [KV(k, v, 0)], scale=1 / math.sqrt(8))
    assert np.array_equal(O1, O2) and np.array_equal(l1, l2)
    # softmax by hand with scipy-free numpy for one row
    s = (f64(q)[0, 0, 0] @ f64(k)[0, 0].T) / math.sqrt(8)
    p = np.exp(s - s.max())
    p /= p.sum()
    assert np.allclose(O1[0, 0, 0], p @ f64(v)[0, 0], atol=1e-14)
    O3, _ = oracle.attention(q, [KV(k, v, 0)], scale=1.0)
    assert not np.allclose(O1, O3)


def test_segment_split_invariance_and_permutation():
    B, Lq, Hq, Hkv, d, Lk = 2, 4, 4, 2, 8, 13
    q, k, v = rnd(30, (B, Lq, Hq, d)), rnd(31, (B, Hkv, Lk, d)), rnd(32, (B, Hkv, Lk, d))
    O, lse = oracle.attention(q, [KV(k, v, 0)])
    for a, b in [(0, 13), (5, 9), (1, 2), (13, 13)]:
        segs = [KV(k[:, :, :a], v[:, :, :a], 0), KV(k[:, :, a:b], v[:, :, a:b], a), KV(k[:, :, b:], v[:, :, b:], b)]
        O2, lse2 = oracle.attention(q, segs)
        assert np.allclose(O, O2, atol=1e-13) and np.allclose(lse, lse2, atol=1e-13)
        O3, _ = oracle.attention(q, segs, mask_mode="block_causal", bs=4, q_pos0=5)
        O4, _ = oracle.attention(q, [KV(k, v, 0)], mask_mode="block_causal", bs=4, q_pos0=5)
        assert np.allclose(O3, O4, atol=1e-13)
    perm = np.random.default_rng(0).permutation(Lk)
    Op, lsep = oracle.attention(q, [KV(k[:, :, perm], v[:, :, perm], 0)])
    assert np.allclose(O, Op, atol=1e-13) and np.allclose(lse, lsep, atol=1e-13)


def test_block_causal_limits():
    B, L, H, d = 1, 12, 2, 8
    q, k, v = rnd(40, (B, L, H, d)), rnd(41, (B, H, L, d)), rnd(42, (B, H, L, d))
    # bs = 1 -> textbook causal attention, computed here with a dense lower-triangular mask
    O1, _ = oracle.attention(q, [KV(k, v, 0)], mask_mode="block_causal", bs=1)
    s = np.einsum("bihd,bhjd->bhij", f64(q), f64(k)) / math.sqrt(d)
    tri = np.tril(np.ones((L, L), bool))
    s = np.where(tri, s, -np.inf)
    p = np.exp(s - s.max(-1, keepdims=True))
    p /= p.sum(-1, keepdims=True)
    want = np.einsum("bhij,bhjd->bihd", p, f64(v))
    assert np.allclose(O1, want, atol=1e-13)
    # bs >= L -> full
    Of, _ = oracle.attention(q, [KV(k, v, 0)])
    Ob, _ = oracle.attention(q, [KV(k, v, 0)], mask_mode="block_causal", bs=L)
    assert np.array_equal(Of, Ob)
    # bs = 4: row 5 sees keys 0..7 exactly
    O4, _ = oracle.attention(q, [KV(k, v, 0)], mask_mode="block_causal", bs=4)
    Oc, _ = oracle.attention(q[:, 5:6], [KV(k[:, :, :8], v[:, :, :8], 0)])
    assert np.allclose(O4[:, 5], Oc[:, 0], atol=1e-13)
    # absolute positions: the same rows asked as a rollout block with q_pos0
    Or, _ = oracle.attention(q[:, 4:8], [KV(k[:, :, :4], v[:, :, :4], 0), KV(k[:, :, 4:8], v[:, :, 4:8], 4)],
                             mask_mode="block_causal", bs=4, q_pos0=4)
    assert np.allclose(O4[:, 4:8], Or, atol=1e-13)


def test_gqa_equals_mha_on_repeated_heads():
    B, Lq, Hq, Hkv, d, Lk = 2, 3, 6, 2, 8, 7
    q, k, v = rnd(50, (B, Lq, Hq, d)), rnd(51, (B, Hkv, Lk, d)), rnd(52, (B, Hkv, Lk, d))
    O, lse = oracle.attention(q, [KV(k, v, 0)])
    krep, vrep = np.repeat(k, 3, axis=1), np.repeat(v, 3, axis=1)     # head h uses kv head h // 3
    O2, lse2 = oracle.attention(q, [KV(krep, vrep, 0)])
    assert np.array_equal(O, O2) and np.array_equal(lse, lse2)
    # and the interleaved mapping (h % Hkv) is NOT what is computed
    kil, vil = np.tile(k, (1, 3, 1, 1)), np.tile(v, (1, 3, 1, 1))
    O3, _ = oracle.attention(q, [KV(kil, vil, 0)])
    assert not np.allclose(O, O3)


def test_cached_equals_full_recompute():
    """Rows [P, P+Lb) of a full-sequence pass equal the rollout call with the exact cache."""
    B, L, Hq, Hkv, d, P, Lb = 2, 20, 4, 2, 8, 9, 4
    q, k, v = rnd(60, (B, L, Hq, d)), rnd(61, (B, Hkv, L, d)), rnd(62, (B, Hkv, L, d))
    Ofull, lfull = oracle.attention(q, [KV(k, v, 0)])
    segs = [KV(k[:, :, :P], v[:, :, :P], 0), KV(k[:, :, P:P + Lb], v[:, :, P:P + Lb], P),
            KV(k[:, :, P + Lb:], v[:, :, P + Lb:], P + Lb)]
    Oc, lc = oracle.attention(q[:, P:P + Lb], segs, q_pos0=P)
    assert np.allclose(Ofull[:, P:P + Lb], Oc, atol=1e-13)
    assert np.allclose(lfull[:, :, P:P + Lb], lc, atol=1e-13)
    # block-causal: prefix + block only (no suffix) == rows of the full block-causal pass
    P2 = 8
    Obc, _ = oracle.attention(q, [KV(k, v, 0)], mask_mode="block_causal", bs=4)
    Or, _ = oracle.attention(q[:, P2:P2 + 4], [KV(k[:, :, :P2], v[:, :, :P2], 0),
                                                KV(k[:, :, P2:P2 + 4], v[:, :, P2:P2 + 4], P2)],
                             mask_mode="block_causal", bs=4, q_pos0=P2)
    assert np.allclose(Obc[:, P2:P2 + 4], Or, atol=1e-13)


def test_two_chunk_lse_merge():
    B, Lq, H, d, Lk = 1, 2, 2, 8, 10
    q, k, v = rnd(70, (B, Lq, H, d)), rnd(71, (B, H, Lk, d)), rnd(72, (B, H, Lk, d))
    O, lse = oracle.attention(q, [KV(k, v, 0)])
    Oa, la = oracle.attention(q, [KV(k[:, :, :6], v[:, :, :6], 0)])
    Ob, lb = oracle.attention(q, [KV(k[:, :, 6:], v[:, :, 6:], 6)])
    la_, lb_ = la.transpose(0, 2, 1)[..., None], lb.transpose(0, 2, 1)[..., None]
    m = np.maximum(la_, lb_)
    wa, wb = np.exp(la_ - m), np.exp(lb_ - m)
    assert np.allclose(O, (wa * Oa + wb * Ob) / (wa + wb), atol=1e-13)
    assert np.allclose(lse.transpose(0, 2, 1)[..., None], m + np.log(wa + wb), atol=1e-13)


def test_rows_subset_and_empty_context():
    B, Lq, Hq, Hkv, d, Lk = 2, 3, 4, 2, 8, 5
    q, k, v = rnd(80, (B, Lq, Hq, d)), rnd(81, (B, Hkv, Lk, d)), rnd(82, (B, Hkv, Lk, d))
    O, lse = oracle.attention(q, [KV(k, v, 0)])
    rows = np.array([[1, 3, 2], [0, 0, 0], [1, 2, 1]], np.int32)
    Or, lr = oracle.attention(q, [KV(k, v, 0)], rows=rows)
    for n, (b, h, i) in enumerate(rows):
        assert np.array_equal(Or[n], O[b, i, h]) and lr[n] == lse[b, h, i]
    # a query that sees nothing: output 0, lse -inf
    O0, l0 = oracle.attention(q, [KV(k, v, 0)], prefix_len_b=np.array([0, 5], np.int32))
    assert np.all(O0[0] == 0) and np.all(np.isinf(l0[0])) and np.array_equal(O0[1], O[1])


def test_bf16_bits_are_read_exactly():
    # 1.00390625 = 1 + 2^-8 is not a bf16; 1.0078125 = 1 + 2^-7 is.  One key, V = that value.
    val = np.array([[[[1.0078125] * 4]]], np.float32)
    v = synth.f32_to_bf16_bits(val)
    q = synth.f32_to_bf16_bits(np.ones((1, 1, 1, 4), np.float32))
    O, _ = oracle.attention(q, [KV(v, v, 0)])
    assert np.all(O == 1.0078125)
    assert bf16_to_float(v.ravel()[0]) == 1.0078125
