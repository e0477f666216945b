"""Generator determinism, bf16 rounding and distribution checks (CPU only)."""
import struct

import numpy as np

from paper_2604_04215_amd import synth


def _rne_bits_reference(f):
    """bit-twiddled round-to-nearest-even of one float32, written independently."""
    (u,) = struct.unpack("<I", struct.pack("<f", f))
    lower = u & 0xFFFF
    upper = u >> 16
    if lower > 0x8000 or (lower == 0x8000 and (upper & 1)):
        upper += 1
    return upper & 0xFFFF


def test_bf16_rounding_matches_bit_reference():
    rng = np.random.default_rng(0)
    x = rng.standard_normal(1 << 16).astype(np.float32) * np.float32(3.0)
    # add exact ties and neighbours
    ties = (np.arange(0x3F80, 0x3F80 + 512, dtype=np.uint32) << 16) | np.uint32(0x8000)
    x = np.concatenate([x, ties.view(np.float32), (ties + 1).view(np.float32), (ties - 1).view(np.float32)])
    got = synth.f32_to_bf16_bits(x)
    want = np.array([_rne_bits_reference(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want)


def test_bf16_roundtrip_exact():
    u = np.arange(0, 1 << 16, dtype=np.uint32).astype(np.uint16)
    f = synth.bf16_bits_to_f32(u)
    ok = ~np.isnan(f)
    assert np.array_equal(synth.f32_to_bf16_bits(f[ok]), u[ok])
    assert np.array_equal(synth.bf16_bits_to_f64(u[ok]), f[ok].astype(np.float64))


def test_per_sequence_independence_of_batch():
    cfg = synth.CONFIGS["mini3"]
    full = synth.step_q(cfg, 1, 2)
    sub = synth.step_q(cfg, 1, 2, seqs=[2])
    assert np.array_equal(full[2], sub[0])
    k, v = synth.cache_kv(cfg, 1)
    k2, v2 = synth.cache_kv(cfg, 1, seqs=[1, 2])
    assert np.array_equal(k[1:], k2) and np.array_equal(v[1:], v2)
    assert not np.array_equal(k, v)
    assert not np.array_equal(synth.step_q(cfg, 1, 2), synth.step_q(cfg, 1, 3))


def test_w_chunking_is_invisible():
    cfg = synth.CONFIGS["mini4"].replace(V=2500)
    w = synth.w_vocab(cfg)
    assert w.shape == (2500, cfg.Dh)
    assert np.array_equal(synth.w_vocab(cfg, slice(1000, 2100)), w[1000:2100])
    assert np.array_equal(synth.w_vocab(cfg, slice(1024, 2048)), w[1024:2048])


def test_moments():
    cfg = synth.CONFIGS["mini2"]
    q = synth.bf16_bits_to_f64(synth.step_q(cfg, 0, 0))
    n = q.size
    assert abs(q.mean()) < 4 / np.sqrt(n)
    assert abs(q.var() - 1.0) < 4 * np.sqrt(2.0 / n) + 1e-3      # bf16 rounding adds ~1e-5 relative
    w = synth.bf16_bits_to_f64(synth.w_vocab(cfg))
    assert abs(w.var() / cfg.Dh ** -0.5 - 1.0) < 0.02            # variance reading: var = Dh^-1/2
    w2 = synth.bf16_bits_to_f64(synth.w_vocab(cfg.replace(w_dist="std")))
    assert abs(w2.std() / cfg.Dh ** -0.5 - 1.0) < 0.02


def test_masks():
    c1 = synth.CONFIGS["c1"]
    m = synth.initial_block_mask(c1, 0)
    assert m.shape == (1, 32) and m.sum() == 16
    assert np.array_equal(m, synth.initial_block_mask(c1, 0))
    assert synth.initial_block_mask(synth.CONFIGS["mini2"], 1).all()
    f = synth.FULLPASS["mini5b"].replace(L=4096, B=4)
    fm = synth.fullpass_mask(f)
    # Eq. (1): i.i.d. masking with probability 1 - alpha_t = 0.5
    assert abs(fm.mean() - 0.5) < 4 * 0.5 / np.sqrt(fm.size)
    x = synth.initial_tokens(f, f.L)
    assert x.dtype == np.int32 and x.min() >= 0 and x.max() < f.V - 1


def test_config_shapes():
    c = synth.CONFIGS
    assert c["c2"].n_blocks == 8 and c["c3"].n_blocks == 16 and c["c4"].Hq // c["c4"].Hkv == 7
    assert c["c5a"].prompt + c["c5a"].gen == 4096
    for name in ("c1", "c2", "c3", "c4", "c5a"):
        assert c[name].V % 256 == 0
