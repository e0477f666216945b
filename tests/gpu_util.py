"""Helpers shared by the GPU parity tests (host <-> device plumbing and error metrics)."""
import numpy as np
import torch

from paper_2604_04215_amd import synth

DEV = "cuda:0"


def bf16_dev(u16: np.ndarray) -> torch.Tensor:
    a = np.ascontiguousarray(u16, dtype=np.uint16)
    return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).to(DEV)


def bf16_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def attn_rel_err(got_u16: np.ndarray, ref: np.ndarray) -> float:
    """max |got - ref| / max(|ref|, rms of the reference row over head_dim): the 2e-2 criterion.

    Why the floor is the row rms: the kernel rounds every probability p_j to bf16 (relative error
    <= 2^-9) before the second product and rounds the output to bf16, so an output element carries an
    absolute error of about 2^-9 * sqrt(sum_j p_j^2 v_jc^2), which scales with the row's typical
    magnitude and not with the element's own value; an element that happens to be near zero has no
    meaningful relative error of its own."""
    got = synth.bf16_bits_to_f64(got_u16).reshape(ref.shape)
    rms = np.sqrt((ref ** 2).mean(axis=-1, keepdims=True))
    den = np.maximum(np.abs(ref), rms)
    den = np.where(den == 0, 1.0, den)
    return float((np.abs(got - ref) / den).max()) if ref.size else 0.0


def attn_err_report(got_u16: np.ndarray, ref: np.ndarray) -> dict:
    """The attention error under every reading of "max relative error" that has been proposed for it:
    rms_floor   max |d| / max(|ref|, row rms)            the pass criterion (attn_rel_err)
    floor_005   max |d| / max(|ref|, 0.05 row rms)       a tighter floor (no bf16-P kernel can meet 2e-2 under
                                                         it: tests/test_attn_error_model.py)
    global      max |d| / max |ref|                      error relative to the largest output
    plain_big   max |d| / |ref| over |ref| >= row rms    the plain relative error where it is meaningful"""
    got = synth.bf16_bits_to_f64(got_u16).reshape(ref.shape)
    if ref.size == 0:
        return dict(rms_floor=0.0, floor_005=0.0, **{"global": 0.0}, plain_big=0.0)
    d = np.abs(got - ref)
    a = np.abs(ref)
    rms = np.sqrt((ref ** 2).mean(axis=-1, keepdims=True))
    one = lambda den: float((d / np.where(den == 0, 1.0, den)).max())
    big = a >= rms
    return {"rms_floor": one(np.maximum(a, rms)), "floor_005": one(np.maximum(a, 0.05 * rms)),
            "global": float(d.max() / max(a.max(), 1e-300)),
            "plain_big": float((d[big] / a[big]).max()) if big.any() and a[big].min() > 0 else 0.0}


def fmt_err(rep: dict) -> str:
    return " ".join(f"{k}={v:.2e}" for k, v in rep.items())


class GuardedWorkspace:
    """A workspace of exactly n bytes with a 4 KB patterned guard band on either side: a kernel that writes one
    byte before or past its workspace changes the pattern, which check() reports."""
    GUARD = 4096

    def __init__(self, nbytes: int):
        n = max(16, (int(nbytes) + 15) // 16 * 16)
        self.raw = torch.empty(n + 2 * self.GUARD, dtype=torch.uint8, device=DEV)
        self.pattern = (torch.arange(self.GUARD, device=DEV) * 37 + 11).to(torch.uint8)
        self.raw[:self.GUARD] = self.pattern
        self.raw[self.GUARD + n:] = self.pattern
        self.ws = self.raw[self.GUARD:self.GUARD + n]      # 16-byte aligned: the guard is a multiple of 256

    def check(self) -> None:
        torch.cuda.synchronize()
        n = self.ws.numel()
        assert torch.equal(self.raw[:self.GUARD], self.pattern), "write before the workspace"
        assert torch.equal(self.raw[self.GUARD + n:], self.pattern), "write past the workspace"


def rnd(seed, shape, std=1.0):
    return synth.normal_bf16(99, 31, (seed,), shape, std)
