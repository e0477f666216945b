"""Which "relative error" a bf16-probability attention kernel can meet (CPU only).

The attention contract is "max relative error 2e-2, bf16 operands with fp32 accumulation".  Any kernel that
feeds the second product (P V) to bf16 matrix units rounds every probability to 8 significant bits and rounds
the output to bf16.  This test plants exactly those two roundings into the oracle's own formula (everything
else in float64) and measures the error of the result against the unrounded oracle under the candidate
readings of "relative":
  * |d| / max(|ref|, row rms)        -> about 8e-3: the 2e-2 bound holds with margin (the criterion in use);
  * |d| / max(|ref|, 0.05 row rms)   -> far above 2e-2: elements that happen to be near zero carry the
    row's absolute error, so no kernel with bf16 probabilities can meet 2e-2 under that floor;
  * max|d| / max|ref| (global)       -> about 1e-3, reported beside the others.
So the row-rms floor is the tightest of the readings that the arithmetic the contract itself prescribes can
satisfy, and it is derived from that arithmetic, not from the HIP kernel (nothing here touches it)."""
import numpy as np

import oracle
from oracle import KV
from paper_2604_04215_amd import synth
from gpu_util import attn_err_report


def bf16_round(x):
    return synth.bf16_bits_to_f64(synth.f32_to_bf16_bits(np.asarray(x, np.float32)))


def emulate_bf16_p(q, k, v, d):
    """softmax(Q K^T / sqrt(d)) V with P and O rounded to bf16, everything else float64."""
    qf, kf, vf = (synth.bf16_bits_to_f64(t) for t in (q, k, v))
    s = np.einsum("bihd,bhjd->bhij", qf, kf) / np.sqrt(d)
    p = np.exp(s - s.max(-1, keepdims=True))
    l = p.sum(-1, keepdims=True)                       # the row sum uses the unrounded probabilities
    o = np.einsum("bhij,bhjd->bihd", bf16_round(p), vf) / l.transpose(0, 2, 1, 3)
    return synth.f32_to_bf16_bits(o.astype(np.float32))


def test_bf16_probabilities_meet_2e2_only_under_the_row_rms_floor():
    reports = []
    for name in ("c1", "mini2", "mini4"):
        cfg = synth.CONFIGS[name]
        o = oracle.OracleRollout(cfg, synth)
        o.begin_block(0)
        q = synth.step_q(cfg, 0, 0)
        kb, vb = synth.step_kv(cfg, 0, 0)
        segs = o.segments(kb, vb)
        ref, _ = oracle.attention(q, segs)
        k = np.concatenate([s.k for s in segs], axis=2)
        v = np.concatenate([s.v for s in segs], axis=2)
        g = cfg.Hq // cfg.Hkv
        got = emulate_bf16_p(q, np.repeat(k, g, axis=1), np.repeat(v, g, axis=1), cfg.d)
        rep = attn_err_report(got, ref)
        reports.append((name, rep))
        assert rep["rms_floor"] <= 2e-2, (name, rep)          # the criterion the GPU tests use is attainable ...
        assert rep["rms_floor"] >= 1e-3, (name, rep)          # ... and not vacuous: the roundings are visible in it
        assert rep["floor_005"] > 2e-2, (name, rep)           # the 0.05 rms floor is not attainable with bf16 P
        assert rep["global"] <= 5e-3, (name, rep)
    print(reports)


def test_error_metric_sees_a_dropped_key_when_attention_is_peaked():
    """The floor does not make the metric blind: leaving one key out of a row whose attention is concentrated on it
    gives an error two orders of magnitude above the bound."""
    rng = np.random.default_rng(5)
    B, Lq, H, d, Lk = 1, 4, 2, 64, 48
    q = synth.f32_to_bf16_bits(rng.standard_normal((B, Lq, H, d)).astype(np.float32))
    k = synth.f32_to_bf16_bits(rng.standard_normal((B, H, Lk, d)).astype(np.float32))
    v = synth.f32_to_bf16_bits(rng.standard_normal((B, H, Lk, d)).astype(np.float32))
    k[:, :, 17] = synth.f32_to_bf16_bits(4.0 * synth.bf16_bits_to_f32(q[:, 0]))     # row 0 attends to key 17
    ref, _ = oracle.attention(q, [KV(k, v, 0)])
    keep = np.arange(Lk) != 17
    dropped, _ = oracle.attention(q, [KV(k[:, :, keep], v[:, :, keep], 0)])
    rep = attn_err_report(synth.f32_to_bf16_bits(dropped.astype(np.float32)), ref)
    assert rep["rms_floor"] > 0.5, rep
