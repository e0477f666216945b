"""dlm_lmhead_confidence_static (the entry point that allocates nothing) against dlm_lmhead_confidence
with a caller-owned workspace: same kernels, same summation order, so every output is identical (GPU)."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2604_04215_amd import binding as dlm
from gpu_util import DEV, bf16_dev, rnd

pytestmark = pytest.mark.gpu


def run_both(M, V, Dh, seed, sample_seed=None, use_rows=False):
    h = bf16_dev(rnd(seed, (M + 7, Dh)))
    w = bf16_dev(rnd(seed + 1, (V, Dh), std=Dh ** -0.25))
    row_idx = None
    if use_rows:
        row_idx = torch.from_numpy(np.random.default_rng(seed).permutation(M + 7)[:M].astype(np.int32)).to(DEV)
    outs = []
    for static in (False, True):
        conf = torch.full((M,), -7.0, device=DEV)
        tok = torch.full((M,), -7, dtype=torch.int32, device=DEV)
        lse, zmax, z2nd = (torch.full((M,), -7.0, device=DEV) for _ in range(3))
        ws = None
        if not static:
            ws = torch.empty(dlm.lmhead_workspace_bytes(M, V, sample=sample_seed is not None), dtype=torch.uint8, device=DEV)
        dlm.lmhead_confidence(h, w, conf, tok, M=M, row_idx=row_idx, forbid_token=V - 1, lse=lse, zmax=zmax, z2nd=z2nd,
                              workspace=ws, sample_seed=sample_seed, sample_step=3, sample_stream=1,
                              static_scratch=static)
        torch.cuda.synchronize()
        outs.append([t.cpu().numpy() for t in (conf, tok, lse, zmax, z2nd)])
    for a, b in zip(*outs):
        assert np.array_equal(a, b)
    assert (outs[1][1] >= 0).all() and (outs[1][1] < V - 1).all()
    assert ((outs[1][0] > 0) & (outs[1][0] <= 1 + 1e-6)).all()


def test_static_scratch_matches_workspace_two_calls_in_a_row():
    """Two calls in a row on the shared scratch, the second smaller (fewer rows, fewer vocabulary tiles): what the
    first left behind must not leak into the second."""
    assert dlm.lib().dlm_lmhead_static_scratch_bytes() == 32 << 20
    run_both(M=300, V=5000, Dh=256, seed=11, use_rows=True)
    run_both(M=37, V=1111, Dh=128, seed=12)
    run_both(M=130, V=4097, Dh=192, seed=13, sample_seed=0xABCDEF)
    run_both(M=5, V=300, Dh=64, seed=14, sample_seed=0xABCDEF, use_rows=True)


def test_static_scratch_rejects_sizes_beyond_its_limit():
    a = dlm.LmheadArgs()
    a.struct_size = C.sizeof(dlm.LmheadArgs)
    M, V, Dh = 4096, 200000, 64                      # 4096 rows x 1563 tiles x 16 B = 102 MB of partials
    h = torch.zeros((M, Dh), dtype=torch.bfloat16, device=DEV)
    w = torch.zeros((V, Dh), dtype=torch.bfloat16, device=DEV)
    conf = torch.zeros(M, device=DEV)
    tok = torch.zeros(M, dtype=torch.int32, device=DEV)
    with pytest.raises(dlm.DlmError) as e:
        dlm.lmhead_confidence(h, w, conf, tok, static_scratch=True)
    assert e.value.code == dlm.DLM_ERR_WORKSPACE and "scratch" in str(e.value)
