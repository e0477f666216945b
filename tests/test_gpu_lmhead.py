"""dlm_lmhead_confidence against the oracle (GPU)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_04215_amd import binding as dlm
from paper_2604_04215_amd import synth
from gpu_util import DEV, GuardedWorkspace, bf16_dev, dev, rnd

pytestmark = pytest.mark.gpu

CONF_TOL = 1e-3     # absolute, confidences
MARGIN = 1e-3       # rows whose top-2 logit margin is below this may legitimately pick the other token
Z_TOL = 2e-3        # logits-scale outputs (lse, zmax, z2nd): fp32 accumulation over Dh terms


def run_lm(hidden, w, *, row_idx=None, M=None, m_dev=None, forbid=-1, inv_t=1.0, scatter=False, target=None,
           M_expected=0):
    R, Dh = hidden.shape
    V = w.shape[0]
    hd, wd = bf16_dev(hidden), bf16_dev(w)
    ridx = None if row_idx is None else dev(np.asarray(row_idx, np.int32))
    Mh = M if M is not None else (len(row_idx) if row_idx is not None else R)
    n_out = R if scatter else Mh
    f = lambda: torch.full((n_out,), float("nan"), dtype=torch.float32, device=DEV)
    conf, lse, zmax, z2nd = f(), f(), f(), f()
    tok = torch.full((n_out,), -7, dtype=torch.int32, device=DEV)
    tgt = zt = None
    if target is not None:
        tgt, zt = dev(np.asarray(target, np.int32)), f()
    gw = GuardedWorkspace(dlm.lmhead_workspace_bytes(Mh, V))     # exactly the size the library asks for, guarded
    dlm.lmhead_confidence(hd, wd, conf, tok, M=Mh, row_idx=ridx,
                          m_dev=None if m_dev is None else dev(np.asarray([m_dev], np.int32)),
                          forbid_token=forbid, inv_temperature=inv_t, out_scatter=scatter,
                          lse=lse, zmax=zmax, z2nd=z2nd, target=tgt, ztarget=zt, workspace=gw.ws,
                          M_expected=M_expected)
    gw.check()
    out = dict(conf=conf.cpu().numpy(), tok=tok.cpu().numpy(), lse=lse.cpu().numpy(), zmax=zmax.cpu().numpy(),
               z2nd=z2nd.cpu().numpy())
    if zt is not None:
        out["zt"] = zt.cpu().numpy()
    return out


def compare_prefix(got, ref, m):
    """The first m outputs against the oracle's; the rest must be untouched.  Few rows: confidences only."""
    if m >= 20:
        compare({k: v[:m] for k, v in got.items()}, {k: v[:m] for k, v in ref.items() if k != "zt"})
    elif m > 0:
        assert np.abs(got["conf"][:m].astype(np.float64) - ref["conf"][:m]).max() <= CONF_TOL
        assert np.abs(got["lse"][:m] - ref["lse"][:m]).max() <= Z_TOL
    assert np.all(np.isnan(got["conf"][m:])) and np.all(got["tok"][m:] == -7)


def compare(got, ref, sel=None):
    """got arrays indexed by output slot; ref from the oracle in the same order (sel picks got's slots)."""
    g = {k: (v if sel is None else v[sel]) for k, v in got.items()}
    assert np.abs(g["conf"].astype(np.float64) - ref["conf"]).max() <= CONF_TOL
    margin = ref["zmax"] - ref["z2nd"]
    clear = margin >= MARGIN
    assert np.array_equal(g["tok"][clear], ref["tok"][clear])
    assert clear.mean() > 0.9
    assert np.abs(g["lse"] - ref["lse"]).max() <= Z_TOL
    assert np.abs(g["zmax"] - ref["zmax"]).max() <= Z_TOL
    both = np.isfinite(ref["z2nd"])
    assert np.abs(g["z2nd"][both] - ref["z2nd"][both]).max() <= Z_TOL
    if "zt" in ref:
        fin = np.isfinite(ref["zt"])
        assert np.abs(g["zt"][fin] - ref["zt"][fin]).max() <= Z_TOL
        assert np.array_equal(np.isfinite(g["zt"]), fin)


@pytest.mark.parametrize("M,Dh,V", [(1, 64, 300), (16, 256, 2048), (33, 128, 777), (64, 192, 1000), (90, 128, 600),
                                    (100, 320, 1500), (150, 128, 700), (200, 256, 900), (256, 128, 2048),
                                    (300, 64, 515), (700, 64, 400)])
def test_shapes_vs_oracle(M, Dh, V):
    # covers every row-tile variant (<=32, <=64, <=128, <=256 rows), several row chunks, ragged V tails
    h, w = rnd(M + Dh, (M, Dh)), rnd(V + Dh, (V, Dh), Dh ** -0.25)
    ref = oracle.lmhead(h, w, forbid_token=V - 1)
    got = run_lm(h, w, forbid=V - 1)
    compare(got, ref)
    assert np.all(got["tok"] != V - 1)


@pytest.mark.parametrize("variant", range(29))
def test_every_kernel_shape(variant):
    # each entry of the library's shape table on a problem with several row chunks and ragged tails
    M, Dh, V = 300, 192, 1100
    h, w = rnd(900, (M, Dh)), rnd(901, (V, Dh), Dh ** -0.25)
    tgt = np.random.default_rng(2).integers(0, V, size=M).astype(np.int32)
    ref = oracle.lmhead(h, w, forbid_token=V - 1, target=tgt)
    dlm.set_option("lmhead_variant", variant)
    try:
        got = run_lm(h, w, forbid=V - 1, target=tgt)
    finally:
        dlm.set_option("lmhead_variant", -1)
    compare(got, ref)


@pytest.mark.parametrize("variant", list(range(10, 24)) + [27])
@pytest.mark.parametrize("Dh", [640, 704])
def test_ring_shapes_reach_their_steady_state_loop(variant, Dh):
    # the direct-to-LDS shapes run prologue + drain only while Dh < 7 stages of 32: here 20 and 22 stages
    M, V = 270, 600
    h, w = rnd(910 + Dh, (M, Dh)), rnd(911 + Dh, (V, Dh), Dh ** -0.25)
    ref = oracle.lmhead(h, w, forbid_token=3)
    dlm.set_option("lmhead_variant", variant)
    try:
        got = run_lm(h, w, forbid=3)
    finally:
        dlm.set_option("lmhead_variant", -1)
    compare(got, ref)


@pytest.mark.parametrize("variant,M", [(0, 413), (1, 413), (20, 2806), (21, 2900), (3, 1400)])
def test_row_chunk_counts_without_a_divisor(variant, M):
    # 13 / 7 / 11 / 12 row chunks: counts that are prime or have only a small divisor, so the blocks of row chunks that an
    # XCD runs side by side degenerate (one chunk per block, or blocks that do not fill the XCD)
    Dh, V = 128, 600
    h, w = rnd(940 + M, (M, Dh)), rnd(941 + M, (V, Dh), Dh ** -0.25)
    ref = oracle.lmhead(h, w, forbid_token=V - 1)
    dlm.set_option("lmhead_variant", variant)
    try:
        got = run_lm(h, w, forbid=V - 1)
    finally:
        dlm.set_option("lmhead_variant", -1)
    compare(got, ref)


def test_gather_scatter_mdev_temperature_target():
    R, Dh, V = 96, 128, 1000
    h, w = rnd(1, (R, Dh)), rnd(2, (V, Dh), Dh ** -0.25)
    idx = np.array(sorted(np.random.default_rng(0).permutation(R)[:41]), np.int32)
    tgt_dense = np.random.default_rng(1).integers(0, V, size=R).astype(np.int32)
    ref = oracle.lmhead(h, w, row_idx=idx, inv_temperature=0.7, forbid_token=5, target=tgt_dense[idx])
    # compact outputs
    got = run_lm(h, w, row_idx=idx, inv_t=0.7, forbid=5, target=tgt_dense[idx])
    compare(got, ref)
    # dense outputs: slot row_idx[r]; untouched slots keep their fill
    got = run_lm(h, w, row_idx=idx, inv_t=0.7, forbid=5, scatter=True, target=tgt_dense)
    compare(got, ref, sel=idx)
    rest = np.setdiff1d(np.arange(R), idx)
    assert np.all(np.isnan(got["conf"][rest])) and np.all(got["tok"][rest] == -7)
    # device-side row count smaller than the host bound: only the first m rows are produced
    got = run_lm(h, w, row_idx=idx, M=41, m_dev=17, inv_t=0.7, forbid=5)
    compare({k: v[:17] for k, v in got.items()}, {k: v[:17] for k, v in ref.items() if k != "zt"})
    assert np.all(np.isnan(got["conf"][17:])) and np.all(got["tok"][17:] == -7)
    got = run_lm(h, w, row_idx=idx, M=41, m_dev=0)
    assert np.all(np.isnan(got["conf"])) and np.all(got["tok"] == -7)


@pytest.mark.parametrize("R,n_sel,variant", [(400, 300, -1), (900, 700, -1), (300, 230, 21), (300, 230, 20)])
def test_gather_mdev_target_on_the_ring_shapes(R, n_sel, variant):
    """Row gather, a device-side row count, a temperature, a forbidden token and target logits through the
    direct-to-LDS shapes the planner takes above 192 rows (two 192-row chunks, 256-row chunks, one 256-row chunk)."""
    Dh, V = 256, 1300
    h, w = rnd(31 + R, (R, Dh)), rnd(32 + R, (V, Dh), Dh ** -0.25)
    idx = np.array(sorted(np.random.default_rng(3).permutation(R)[:n_sel]), np.int32)
    tgt = np.random.default_rng(4).integers(0, V, size=n_sel).astype(np.int32)
    ref = oracle.lmhead(h, w, row_idx=idx, inv_temperature=1.3, forbid_token=777, target=tgt)
    dlm.set_option("lmhead_variant", variant)
    try:
        got = run_lm(h, w, row_idx=idx, inv_t=1.3, forbid=777, target=tgt)
        compare(got, ref)
        m = n_sel - 37
        got = run_lm(h, w, row_idx=idx, M=n_sel, m_dev=m, inv_t=1.3, forbid=777)
    finally:
        dlm.set_option("lmhead_variant", -1)
    compare({k: v[:m] for k, v in got.items()}, {k: v[:m] for k, v in ref.items() if k != "zt"})
    assert np.all(np.isnan(got["conf"][m:])) and np.all(got["tok"][m:] == -7)
    # far fewer rows on the device than the host's bound: most row tiles of the launch are dead (their wavefronts
    # only take part in the loads and barriers), down to one row and to none
    dlm.set_option("lmhead_variant", variant)
    try:
        for m in (n_sel // 2, 33, 1, 0):
            compare_prefix(run_lm(h, w, row_idx=idx, M=n_sel, m_dev=m, inv_t=1.3, forbid=777), ref, m)
    finally:
        dlm.set_option("lmhead_variant", -1)


@pytest.mark.parametrize("bound,variant", [(100, 3), (128, 3), (192, 4), (250, 5), (256, 21)])
def test_device_row_count_below_the_bound_in_row_split_shapes(bound, variant):
    """Shapes whose wavefronts split the rows run one copy of their loop per count of live row tiles."""
    Dh, V = 320, 900
    h, w = rnd(51 + bound, (bound, Dh)), rnd(52 + bound, (V, Dh), Dh ** -0.25)
    ref = oracle.lmhead(h, w, forbid_token=V - 1)
    dlm.set_option("lmhead_variant", variant)
    try:
        for m in sorted({bound, bound - 31, bound - 32, bound // 2 + 1, 65, 64, 33, 32, 1}, reverse=True):
            if m < 1 or m > bound:
                continue
            compare_prefix(run_lm(h, w, M=bound, m_dev=m, forbid=V - 1), ref, m)
    finally:
        dlm.set_option("lmhead_variant", -1)


def test_non_temporal_w_stream_changes_nothing():
    """One row chunk: W is fetched with non-temporal loads unless the option turns that off; same bits either way."""
    h, w = rnd(71, (150, 256)), rnd(72, (3000, 256), 0.25)
    a = run_lm(h, w, forbid=11)
    dlm.set_option("lmhead_nt", 0)
    try:
        b = run_lm(h, w, forbid=11)
    finally:
        dlm.set_option("lmhead_nt", 1)
    for k in a:
        assert np.array_equal(a[k], b[k])
    with pytest.raises(dlm.DlmError):
        dlm.set_option("lmhead_nt", 2)


def test_extreme_logits_and_tiny_vocabularies():
    """Logits of magnitude ~500 (max-subtracted soft-max must not overflow), a vocabulary of one token, and one of
    two tokens with one of them forbidden (confidence exactly 1)."""
    Dh = 128
    h = synth.f32_to_bf16_bits(np.random.default_rng(1).normal(size=(70, Dh)).astype(np.float32) * 6.0)
    w = synth.f32_to_bf16_bits(np.random.default_rng(2).normal(size=(500, Dh)).astype(np.float32) * 6.0)
    ref = oracle.lmhead(h, w, forbid_token=3)
    assert np.abs(ref["zmax"]).max() > 300
    got = run_lm(h, w, forbid=3)
    assert np.all(np.isfinite(got["conf"])) and np.all(np.isfinite(got["lse"]))
    clear = (ref["zmax"] - ref["z2nd"]) >= 1e-1
    assert np.array_equal(got["tok"][clear], ref["tok"][clear])
    assert np.abs(got["conf"] - ref["conf"])[clear].max() <= 2e-2      # |logit| ~ 500 at bf16-product precision
    assert np.abs(got["lse"] - ref["lse"]).max() <= 1e-3 * np.abs(ref["lse"]).max()
    for V, forbid in ((1, -1), (2, 1), (2, 0)):
        w1 = rnd(7 + V, (V, Dh), 0.3)
        got = run_lm(rnd(8, (40, Dh)), w1, forbid=forbid)
        want_tok = 0 if forbid != 0 else 1
        assert np.all(got["tok"] == want_tok)
        if V == 1 or forbid >= 0:
            assert np.allclose(got["conf"], 1.0, atol=1e-6)
            assert np.all(got["z2nd"] == -np.inf)


def test_ties_pick_lowest_index():
    Dh, V = 64, 700
    h = synth.f32_to_bf16_bits(np.ones((40, Dh), np.float32))
    w = synth.f32_to_bf16_bits(np.full((V, Dh), 0.25, np.float32))
    got = run_lm(h, w)
    assert np.all(got["tok"] == 0)
    assert np.allclose(got["conf"], 1.0 / V, atol=1e-6)
    assert np.allclose(got["z2nd"], got["zmax"])
    got = run_lm(h, w, forbid=0)
    assert np.all(got["tok"] == 1) and np.allclose(got["conf"], 1.0 / (V - 1), atol=1e-6)
    # two equal maxima in different vocabulary tiles: the lower one wins
    wf = np.zeros((V, Dh), np.float32)
    wf[650, 0] = 2.0
    wf[131, 0] = 2.0
    got = run_lm(synth.f32_to_bf16_bits(np.eye(3, Dh, dtype=np.float32)), synth.f32_to_bf16_bits(wf))
    assert got["tok"][0] == 131 and got["z2nd"][0] == got["zmax"][0] == 2.0


def test_closed_form_threshold_boundary():
    # z = (a, 0, ..., 0): conf = e^a / (e^a + V - 1)
    Dh, V = 64, 2048
    for a in (2.0, 7.5, 9.8125):
        wf = np.zeros((V, Dh), np.float32)
        wf[1234, 0] = a
        got = run_lm(synth.f32_to_bf16_bits(np.eye(1, Dh, dtype=np.float32)), synth.f32_to_bf16_bits(wf))
        want = np.exp(a) / (np.exp(a) + V - 1)
        assert got["tok"][0] == 1234 and abs(got["conf"][0] - want) < 1e-5


def test_rerun_is_bitwise_identical():
    h, w = rnd(5, (200, 256)), rnd(6, (3000, 256), 0.25)
    a, b = run_lm(h, w), run_lm(h, w)
    for k in a:
        assert np.array_equal(a[k], b[k])


def test_full_vocabulary_sampled_rows():
    """LLaDA-8B-sized head (V = 126464, Dh = 4096), 256 rows as in the benchmark's first step;
    the oracle checks a sample of rows one by one."""
    cfg = synth.CONFIGS["c2"]
    w = synth.w_vocab(cfg)
    hid = synth.step_hidden(cfg, 0, 0).reshape(cfg.B * cfg.Lb, cfg.Dh)
    got = run_lm(hid, w, forbid=cfg.forbid_token)
    sample = np.array([0, 31, 77, 128, 200, 255], np.int32)
    ref = oracle.lmhead(hid, w, row_idx=sample, forbid_token=cfg.forbid_token)
    g = {k: v[sample] for k, v in got.items()}
    assert np.abs(g["conf"] - ref["conf"]).max() <= CONF_TOL
    clear = (ref["zmax"] - ref["z2nd"]) >= MARGIN
    assert np.array_equal(g["tok"][clear], ref["tok"][clear])
    assert np.abs(g["lse"] - ref["lse"]).max() <= 5e-3 and np.abs(g["zmax"] - ref["zmax"]).max() <= 5e-3
    # properties that hold at any size
    assert np.all(got["conf"] > 0) and np.all(got["conf"] <= 1.0 + 1e-6)
    assert np.all((got["tok"] >= 0) & (got["tok"] < cfg.V - 1))
    assert np.all(got["z2nd"] <= got["zmax"]) and np.all(got["lse"] >= got["zmax"])
    assert np.allclose(got["conf"], np.exp(got["zmax"] - got["lse"]), atol=1e-5)


@pytest.mark.parametrize("variant", [-1, 0, 3, 5, 7, 10, 16, 20, 21])
@pytest.mark.parametrize("mode", ["margin", "neg_entropy"])
def test_alternative_confidence_scores(mode, variant):
    """conf = p(top-1) - p(top-2) or sum_v p_v log p_v instead of the token probability; every other output unchanged."""
    M, Dh, V = 300, 192, 1100
    h, w = rnd(920, (M, Dh)), rnd(921, (V, Dh), Dh ** -0.25)
    ref = oracle.lmhead(h, w, forbid_token=V - 1, inv_temperature=0.8)
    hd, wd = bf16_dev(h), bf16_dev(w)
    cm = dlm.CONF_MARGIN if mode == "margin" else dlm.CONF_NEG_ENTROPY
    conf = torch.full((M,), float("nan"), dtype=torch.float32, device=DEV)
    lse = torch.full((M,), float("nan"), dtype=torch.float32, device=DEV)
    tok = torch.full((M,), -7, dtype=torch.int32, device=DEV)
    ws = torch.empty(dlm.lmhead_workspace_bytes(M, V, conf_mode=cm), dtype=torch.uint8, device=DEV)
    dlm.set_option("lmhead_variant", variant)
    try:
        dlm.lmhead_confidence(hd, wd, conf, tok, forbid_token=V - 1, inv_temperature=0.8, lse=lse, workspace=ws, conf_mode=cm)
        torch.cuda.synchronize()
    finally:
        dlm.set_option("lmhead_variant", -1)
    got = conf.cpu().numpy().astype(np.float64)
    tol = CONF_TOL if mode == "margin" else Z_TOL          # the entropy lives on the logits' scale
    assert np.abs(got - ref[mode]).max() <= tol
    clear = (ref["zmax"] - ref["z2nd"]) >= MARGIN
    assert np.array_equal(tok.cpu().numpy()[clear], ref["tok"][clear])
    assert np.abs(lse.cpu().numpy() - ref["lse"]).max() <= Z_TOL
    if mode == "neg_entropy":
        assert np.all(got <= 1e-4) and np.all(got >= -np.log(V) - 1e-3)


def test_entropy_full_vocabulary_and_sampling_together():
    """LLaDA-sized head: negative entropy on sampled rows; with sampling on, the score is that of the distribution
    while the token is the drawn one."""
    from oracle import sampling
    cfg = synth.CONFIGS["c2"]
    w = synth.w_vocab(cfg)
    hid = synth.step_hidden(cfg, 0, 1).reshape(-1, cfg.Dh)
    idx = np.sort(np.random.default_rng(5).permutation(hid.shape[0])[:70]).astype(np.int32)
    M = len(idx)
    conf = torch.zeros(M, dtype=torch.float32, device=DEV)
    tok = torch.zeros(M, dtype=torch.int32, device=DEV)
    ws = torch.empty(dlm.lmhead_workspace_bytes(M, cfg.V, sample=True, conf_mode=dlm.CONF_NEG_ENTROPY), dtype=torch.uint8, device=DEV)
    dlm.lmhead_confidence(bf16_dev(hid), bf16_dev(w), conf, tok, M=M, row_idx=dev(idx), forbid_token=cfg.forbid_token,
                          workspace=ws, conf_mode=dlm.CONF_NEG_ENTROPY, sample_seed=99, sample_step=4)
    torch.cuda.synchronize()
    pick = np.array([0, 13, 41, 69])
    ref = oracle.lmhead(hid, w, row_idx=idx[pick], forbid_token=cfg.forbid_token)
    smp = sampling.lmhead_sampled(hid, w, seed=99, step=4, row_idx=idx[pick], forbid_token=cfg.forbid_token)
    assert np.abs(conf.cpu().numpy()[pick] - ref["neg_entropy"]).max() <= Z_TOL
    clear = (smp["pmax"] - smp["p2nd"]) >= MARGIN
    assert np.array_equal(tok.cpu().numpy()[pick][clear], smp["tok"][clear])


@pytest.mark.parametrize("M,m_dev,guess", [(256, 120, 125), (256, 130, 125), (256, 128, 128), (256, 129, 100), (200, 40, 60),
                                           (200, 65, 60), (100, 20, 30), (100, 33, 30), (64, 10, 20), (500, 200, 250),
                                           (500, 300, 250), (500, 500, 250), (300, 0, 100), (128, 128, 90), (70, 70, 1)])
def test_expected_row_count_only_selects_the_shape(M, m_dev, guess):
    """M_expected queues the shape for the guessed count, guarded by the device's count, in front of the shape for the
    bound: whether the guess holds (count within that shape's capacity) or not, the outputs are the oracle's and,
    up to the rounding of another summation order, those of a call without a guess."""
    Dh, V = 256, 1500
    h, w = rnd(7100 + M, (M, Dh)), rnd(7200 + M, (V, Dh), Dh ** -0.25)
    idx = np.arange(M - 1, -1, -1).astype(np.int32)            # gathered rows, reversed
    plain = run_lm(h, w, row_idx=idx, M=M, m_dev=m_dev, forbid=V - 1)
    guessed = run_lm(h, w, row_idx=idx, M=M, m_dev=m_dev, forbid=V - 1, M_expected=guess)
    assert np.array_equal(np.isnan(plain["conf"]), np.isnan(guessed["conf"]))
    assert np.allclose(plain["conf"][:m_dev], guessed["conf"][:m_dev], rtol=0, atol=2e-6)
    assert np.allclose(plain["lse"][:m_dev], guessed["lse"][:m_dev], rtol=0, atol=1e-4)
    assert np.array_equal(plain["tok"], guessed["tok"])
    ref = oracle.lmhead(h, w, row_idx=idx[:m_dev], forbid_token=V - 1)
    compare_prefix(guessed, ref, m_dev)


def test_expected_row_count_with_sampling_and_entropy_partials():
    """The second partial array sits at another offset in the guessed shape's layout: sampled tokens and the
    entropy confidence must not depend on the guess either (beyond rounding)."""
    M, Dh, V = 200, 256, 3000
    h, w = bf16_dev(rnd(7301, (M, Dh))), bf16_dev(rnd(7302, (V, Dh), Dh ** -0.25))
    for kw in (dict(sample_seed=11, sample_step=3), dict(conf_mode=dlm.CONF_NEG_ENTROPY)):
        outs = []
        for guess, md in ((0, 50), (60, 50), (60, 70)):
            conf = torch.full((M,), float("nan"), dtype=torch.float32, device=DEV)
            tok = torch.full((M,), -7, dtype=torch.int32, device=DEV)
            ws = torch.empty(dlm.lmhead_workspace_bytes(M, V, sample="sample_seed" in kw, conf_mode=kw.get("conf_mode", dlm.CONF_TOKEN_PROB)),
                             dtype=torch.uint8, device=DEV)
            dlm.lmhead_confidence(h, w, conf, tok, M=M, m_dev=dev(np.asarray([md], np.int32)), workspace=ws,
                                  M_expected=guess, **kw)
            torch.cuda.synchronize()
            outs.append((conf.cpu().numpy(), tok.cpu().numpy()))
        # the same tokens; confidences up to the rounding of another summation order
        assert np.array_equal(outs[0][1], outs[1][1]) and np.array_equal(outs[0][1][:50], outs[2][1][:50])
        assert np.allclose(outs[0][0], outs[1][0], rtol=0, atol=1e-5, equal_nan=True)
        assert np.allclose(outs[0][0][:50], outs[2][0][:50], rtol=0, atol=1e-5)
        assert not np.isnan(outs[2][0][:70]).any() and np.isnan(outs[2][0][70:]).all()


@pytest.mark.parametrize("M,cus,V", [(70, 8, 2600), (100, 8, 2400), (128, 4, 1500), (150, 8, 2561), (192, 8, 2300), (230, 8, 2500),
                                     (256, 6, 2047), (96, 8, 2305)])
def test_half_height_tail_launch(M, cus, V):
    """A vocabulary whose tile count leaves the last round of workgroups at most half full is covered by two launches:
    full-height tiles, then half-height ones for the tail.  The assumed CU count is lowered so that a small problem
    takes that path (e.g. 2600 rows = 11 tiles of 256 on 8 'CUs': 8 full tiles + 5 half tiles, the last one ragged);
    every output against the oracle, with a forbidden token in the tail and targets on both sides of the seam."""
    Dh = 128
    h, w = rnd(1300 + M, (M, Dh)), rnd(1301 + M, (V, Dh), Dh ** -0.25)
    tgt = np.random.default_rng(M).integers(0, V, size=M).astype(np.int32)
    tgt[:4] = [0, V - 2, (V // 256 // cus * cus) * 256 - 1, min(V - 2, (V // 256 // cus * cus) * 256)]   # around the seam
    ref = oracle.lmhead(h, w, forbid_token=V - 1, target=tgt)
    dlm.set_option("lmhead_cus", cus)
    try:
        got = run_lm(h, w, forbid=V - 1, target=tgt)
        compare(got, ref)
        # device-side row count below the bound, and the two-shape queue on top of the two-launch tail
        m_dev = max(1, M - 37)
        got = run_lm(h, w, forbid=V - 1, m_dev=m_dev, M_expected=max(1, int(0.8 * M)))
        compare_prefix(got, ref, m_dev)
    finally:
        dlm.set_option("lmhead_cus", 0)
    # and with the tail rule switched off the same values up to summation order
    dlm.set_option("lmhead_cus", -1)
    try:
        compare(run_lm(h, w, forbid=V - 1, target=tgt), ref)
    finally:
        dlm.set_option("lmhead_cus", 0)
