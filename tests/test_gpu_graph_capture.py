"""The library's calls under HIP graph capture (GPU): they only launch kernels on the caller's stream (no allocation, no
memset, no synchronisation), so a captured step can be replayed; dlm_lmhead_confidence_static exists for exactly such callers.
Every replay is compared with an eager call on the same inputs, with eager work between the replays."""
import numpy as np
import pytest
import torch

from paper_2604_04215_amd import binding as dlm
from gpu_util import DEV, bf16_dev, rnd

pytestmark = pytest.mark.gpu


def test_attention_and_static_lm_head_replayed_from_a_graph():
    B, Lq, Hq, Hkv, d, P = 2, 32, 8, 2, 128, 300
    M, V, Dh = B * Lq, 3000, 256
    q = bf16_dev(rnd(50, (B, Lq, Hq, d)))
    ck, cv = bf16_dev(rnd(51, (B, Hkv, P, d))), bf16_dev(rnd(52, (B, Hkv, P, d)))
    kb, vb = bf16_dev(rnd(53, (B, Hkv, Lq, d))), bf16_dev(rnd(54, (B, Hkv, Lq, d)))
    out = torch.zeros_like(q)
    h = bf16_dev(rnd(55, (M, Dh)))
    w = bf16_dev(rnd(56, (V, Dh), std=Dh ** -0.25))
    conf = torch.zeros(M, device=DEV)
    tok = torch.zeros(M, dtype=torch.int32, device=DEV)

    def step():
        dlm.block_attn(q, out, prefix=(ck, cv, 0), block=(kb, vb, P), suffix=None, mask_mode=dlm.MASK_FULL)
        dlm.lmhead_confidence(h, w, conf, tok, forbid_token=V - 1, static_scratch=True)

    step()                                   # eager first: the first call on a device looks up the scratch address
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        step()                               # the binding passes torch's current stream: the capturing one
    for rep in range(3):
        q.copy_(bf16_dev(rnd(60 + rep, (B, Lq, Hq, d))))          # eager work between replays: new inputs in place
        h.copy_(bf16_dev(rnd(70 + rep, (M, Dh))))
        out.zero_(); conf.fill_(-1.0); tok.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (out, conf, tok)]
        out.zero_(); conf.fill_(-1.0); tok.fill_(-1)
        step()
        torch.cuda.synchronize()
        for a, b in zip(got, (out, conf, tok)):
            assert torch.equal(a, b), f"replay {rep} differs from the eager call"
        assert float(conf.min()) > 0 and int(tok.min()) >= 0
