"""Logits-free masked log-likelihood: dlm_lmhead_confidence(target) -> dlm_seq_logprob against the oracle (GPU)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_04215_amd import binding as dlm
from gpu_util import DEV, bf16_dev, dev, rnd

pytestmark = pytest.mark.gpu

TERM_TOL = 4e-3    # per masked position: two logits-scale fp32 outputs (target logit, LSE), 2e-3 each


def gpu_seq_logprob(h, w, tgt, mask, weight=None, forbid=-1):
    B, n, Dh = h.shape
    V = w.shape[0]
    hd, wd = bf16_dev(h.reshape(B * n, Dh)), bf16_dev(w)
    md = dev(mask)
    row_idx = torch.empty(B * n, dtype=torch.int32, device=DEV)
    m_out = torch.zeros(1, dtype=torch.int32, device=DEV)
    dlm.mask_compact(md, row_idx, m_out)
    M = int(m_out.item())
    assert M == int(mask.sum())
    f = lambda: torch.full((B * n,), float("nan"), dtype=torch.float32, device=DEV)
    conf, lse, zt = f(), f(), f()
    tok = torch.zeros(B * n, dtype=torch.int32, device=DEV)
    out = torch.full((B,), float("nan"), dtype=torch.float32, device=DEV)
    cnt = torch.full((B,), -1, dtype=torch.int32, device=DEV)
    if M:
        ws = torch.empty(max(16, dlm.lmhead_workspace_bytes(M, V)), dtype=torch.uint8, device=DEV)
        dlm.lmhead_confidence(hd, wd, conf, tok, M=M, row_idx=row_idx, forbid_token=forbid, out_scatter=True,
                              lse=lse, target=dev(tgt.reshape(-1).astype(np.int32)), ztarget=zt, workspace=ws)
    dlm.seq_logprob(zt, lse, md, out, weight=None if weight is None else dev(np.asarray(weight, np.float32)),
                    n_terms=cnt)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64), cnt.cpu().numpy()


@pytest.mark.parametrize("B,n,Dh,V,forbid,weighted", [
    (4, 96, 256, 1000, -1, False),      # ragged vocabulary tail
    (3, 300, 128, 4096, 4095, True),    # more positions than one pass of the reduction's threads
    (1, 1, 64, 200, -1, False),
    (5, 33, 512, 2304, -1, True),
])
def test_matches_oracle(B, n, Dh, V, forbid, weighted):
    h, w = rnd(21, (B, n, Dh)), rnd(22, (V, Dh), Dh ** -0.5)
    g = np.random.default_rng(B * 1000 + n)
    tgt = g.integers(0, V - 1, (B, n))
    mask = (g.random((B, n)) < 0.6).astype(np.uint8)
    if B > 1:
        mask[1] = 0                      # a sequence with nothing masked
    weight = -1.0 / g.uniform(0.1, 1.0, B) if weighted else None
    want, want_cnt = oracle.seq_logprob(h, w, tgt, mask, weight=weight, forbid_token=forbid)
    got, cnt = gpu_seq_logprob(h, w, tgt, mask, weight, forbid)
    assert np.array_equal(cnt, want_cnt)
    scale = np.abs(weight) if weighted else np.ones(B)
    tol = TERM_TOL * np.maximum(want_cnt, 1) * scale + 1e-6 * np.abs(want)
    assert np.all(np.abs(got - want) <= tol), (got, want)
    if B > 1:
        assert got[1] == 0.0


def test_strided_mask_and_determinism():
    B, n = 6, 777
    g = np.random.default_rng(5)
    zt = torch.from_numpy(g.normal(size=(B, n)).astype(np.float32)).to(DEV)
    lse = torch.from_numpy((g.normal(size=(B, n)) + 9).astype(np.float32)).to(DEV)
    big = torch.from_numpy((g.random((B, 2 * n)) < 0.5).astype(np.uint8)).to(DEV)
    mask = big[:, 5:5 + n]
    outs = []
    for _ in range(3):
        out = torch.empty(B, dtype=torch.float32, device=DEV)
        dlm.seq_logprob(zt, lse, mask, out)
        outs.append(out.cpu().numpy())
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])
    m = mask.cpu().numpy().astype(np.float64)
    want = ((zt.cpu().numpy().astype(np.float64) - lse.cpu().numpy().astype(np.float64)) * m).sum(1)
    assert np.abs(outs[0] - want).max() <= 1e-6 * n * 10


def test_rejects_bad_arguments():
    z = torch.zeros(8, dtype=torch.float32, device=DEV)
    m = torch.ones((2, 4), dtype=torch.uint8, device=DEV)
    with pytest.raises(ValueError):
        dlm.seq_logprob(z[:6], z, m, z[:2])
    rc = dlm.lib().dlm_seq_logprob(z.data_ptr(), z.data_ptr(), m.data_ptr(), 2, None, 2, 4, z.data_ptr(), None, None)
    assert rc == dlm.DLM_ERR_INVALID_ARG      # mask row stride below n_pos
