"""ctypes binding to libdlm.so: argument marshalling only.

Every function here fills the C structs of include/dlm.h from torch tensors
(device pointers, element strides) and calls the library on the current torch
HIP stream.  There is no fallback: if the HIP library has not been built, or a
tensor is not on the GPU, the call raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdlm.so")

SEG_CAUSAL, SEG_EARLIER_BLOCKS, SEG_SAME_BLOCK = 0, 1, 2
DLM_OK, DLM_ERR_INVALID_ARG, DLM_ERR_UNSUPPORTED, DLM_ERR_WORKSPACE, DLM_ERR_HIP = 0, -1, -2, -3, -4
MASK_FULL, MASK_BLOCK_CAUSAL = 0, 1
RULE_THRESHOLD, RULE_TOPK = 0, 1
CONF_TOKEN_PROB, CONF_MARGIN, CONF_NEG_ENTROPY = 0, 1, 2
WB_NONE, WB_BLOCK_WHEN_DONE, WB_COMMITTED_ROWS, WB_WHILE_ACTIVE = 0, 1, 2, 3

EXPORTS = ["dlm_block_attn", "dlm_block_attn_workspace_bytes", "dlm_lmhead_confidence",
           "dlm_lmhead_workspace_bytes", "dlm_lmhead_confidence_static", "dlm_lmhead_static_scratch_bytes", "dlm_unmask_commit", "dlm_mask_compact", "dlm_kv_refresh",
           "dlm_block_attn_bwd", "dlm_block_attn_bwd_workspace_bytes", "dlm_seq_logprob", "dlm_set_option", "dlm_last_error", "dlm_version"]


class KvSeg(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("len", C.c_int32), ("pos0", C.c_int32),
                ("stride_b", C.c_int64), ("stride_h", C.c_int64), ("stride_t", C.c_int64), ("rule", C.c_int32)]


class AttnArgs(C.Structure):
    _fields_ = [("struct_size", C.c_uint32),
                ("B", C.c_int32), ("Lq", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("d", C.c_int32),
                ("q", C.c_void_p), ("q_stride_b", C.c_int64), ("q_stride_t", C.c_int64), ("q_stride_h", C.c_int64),
                ("prefix", KvSeg), ("block", KvSeg), ("suffix", KvSeg),
                ("prefix_len_b", C.c_void_p),
                ("mask_mode", C.c_int32), ("block_size", C.c_int32), ("q_pos0", C.c_int32), ("scale", C.c_float),
                ("out", C.c_void_p), ("o_stride_b", C.c_int64), ("o_stride_t", C.c_int64), ("o_stride_h", C.c_int64),
                ("lse", C.c_void_p), ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
                ("cu_seqlens", C.c_void_p), ("total_tokens", C.c_int32), ("seq_active", C.c_void_p)]


class AttnBwdArgs(C.Structure):
    _fields_ = [("struct_size", C.c_uint32),
                ("B", C.c_int32), ("Lq", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("d", C.c_int32),
                ("q", C.c_void_p), ("q_stride_b", C.c_int64), ("q_stride_t", C.c_int64), ("q_stride_h", C.c_int64),
                ("out", C.c_void_p), ("o_stride_b", C.c_int64), ("o_stride_t", C.c_int64), ("o_stride_h", C.c_int64),
                ("d_out", C.c_void_p), ("do_stride_b", C.c_int64), ("do_stride_t", C.c_int64), ("do_stride_h", C.c_int64),
                ("lse", C.c_void_p),
                ("prefix", KvSeg), ("block", KvSeg), ("suffix", KvSeg),
                ("mask_mode", C.c_int32), ("block_size", C.c_int32), ("q_pos0", C.c_int32), ("scale", C.c_float),
                ("d_q", C.c_void_p), ("dq_stride_b", C.c_int64), ("dq_stride_t", C.c_int64), ("dq_stride_h", C.c_int64),
                ("d_prefix_k", C.c_void_p), ("d_prefix_v", C.c_void_p), ("d_block_k", C.c_void_p),
                ("d_block_v", C.c_void_p), ("d_suffix_k", C.c_void_p), ("d_suffix_v", C.c_void_p),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
                ("cu_seqlens", C.c_void_p), ("total_tokens", C.c_int32)]


class LmheadArgs(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("M", C.c_int32), ("Dh", C.c_int32), ("V", C.c_int32),
                ("hidden", C.c_void_p), ("hidden_stride_row", C.c_int64),
                ("row_idx", C.c_void_p), ("m_dev", C.c_void_p),
                ("w", C.c_void_p), ("w_stride_row", C.c_int64),
                ("inv_temperature", C.c_float), ("forbid_token", C.c_int32), ("out_scatter", C.c_int32),
                ("conf", C.c_void_p), ("tok", C.c_void_p),
                ("lse", C.c_void_p), ("zmax", C.c_void_p), ("z2nd", C.c_void_p),
                ("target", C.c_void_p), ("ztarget", C.c_void_p),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
                ("sample", C.c_int32), ("sample_step", C.c_uint32), ("sample_stream", C.c_uint32),
                ("sample_seed", C.c_uint64), ("conf_mode", C.c_int32), ("M_expected", C.c_int32)]


class CommitArgs(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("B", C.c_int32), ("n_pos", C.c_int32), ("group_len", C.c_int32),
                ("rule", C.c_int32), ("threshold", C.c_float), ("force_top1", C.c_int32), ("k", C.c_int32),
                ("conf", C.c_void_p), ("tok", C.c_void_p),
                ("x", C.c_void_p), ("x_stride_b", C.c_int64), ("x_pos0", C.c_int32),
                ("mask", C.c_void_p), ("mask_stride_b", C.c_int64),
                ("commit_now", C.c_void_p), ("n_commit", C.c_void_p), ("remaining", C.c_void_p),
                ("next_row_idx", C.c_void_p), ("next_m", C.c_void_p),
                ("commit_step", C.c_void_p), ("step", C.c_int32), ("writeback", C.c_int32),
                ("src_block", KvSeg), ("cache_k", C.c_void_p), ("cache_v", C.c_void_p),
                ("c_stride_b", C.c_int64), ("c_stride_h", C.c_int64), ("c_stride_t", C.c_int64),
                ("cache_pos0", C.c_int32), ("Hkv", C.c_int32), ("d", C.c_int32),
                ("host_remaining_total", C.c_void_p), ("active_in", C.c_void_p), ("host_remaining_max", C.c_void_p)]


class DlmError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libdlm error {code}: {msg}")
        self.code = code


_lib = None


def lib():
    """Load libdlm.so (built in-tree by paper_2604_04215_amd.build); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not found: build it with `python -m paper_2604_04215_amd.build` "
                               "(there is no CPU fallback)")
        # PyTorch ships its own HIP runtime: load it first so that the library binds to the runtime that owns the
        # tensors' memory and streams (loaded the other way round, launches fail with "no ROCm-capable device")
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        L.dlm_block_attn.restype = C.c_int
        L.dlm_block_attn.argtypes = [C.POINTER(AttnArgs), C.c_void_p]
        L.dlm_block_attn_workspace_bytes.restype = C.c_size_t
        L.dlm_block_attn_workspace_bytes.argtypes = [C.POINTER(AttnArgs)]
        L.dlm_lmhead_confidence.restype = C.c_int
        L.dlm_lmhead_confidence.argtypes = [C.POINTER(LmheadArgs), C.c_void_p]
        L.dlm_lmhead_workspace_bytes.restype = C.c_size_t
        L.dlm_lmhead_workspace_bytes.argtypes = [C.POINTER(LmheadArgs)]
        L.dlm_lmhead_confidence_static.restype = C.c_int
        L.dlm_lmhead_confidence_static.argtypes = [C.POINTER(LmheadArgs), C.c_void_p]
        L.dlm_lmhead_static_scratch_bytes.restype = C.c_size_t
        L.dlm_lmhead_static_scratch_bytes.argtypes = []
        L.dlm_unmask_commit.restype = C.c_int
        L.dlm_unmask_commit.argtypes = [C.POINTER(CommitArgs), C.c_void_p]
        L.dlm_mask_compact.restype = C.c_int
        L.dlm_mask_compact.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.dlm_kv_refresh.restype = C.c_int
        L.dlm_kv_refresh.argtypes = [C.POINTER(KvSeg), C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                     C.c_int64, C.c_int64, C.c_int64, C.c_int32, C.c_void_p]
        L.dlm_block_attn_bwd.restype = C.c_int
        L.dlm_block_attn_bwd.argtypes = [C.c_void_p, C.c_void_p]
        L.dlm_block_attn_bwd_workspace_bytes.restype = C.c_size_t
        L.dlm_block_attn_bwd_workspace_bytes.argtypes = [C.c_void_p]
        L.dlm_seq_logprob.restype = C.c_int
        L.dlm_seq_logprob.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.c_int32,
                                      C.c_void_p, C.c_void_p, C.c_void_p]
        L.dlm_set_option.restype = C.c_int
        L.dlm_set_option.argtypes = [C.c_char_p, C.c_int]
        L.dlm_last_error.restype = C.c_char_p
        L.dlm_version.restype = C.c_int
        _lib = L
    return _lib


def last_error() -> str:
    return lib().dlm_last_error().decode()


def _check(rc: int) -> None:
    if rc != DLM_OK:
        raise DlmError(rc, last_error())


def _stream(stream=None) -> C.c_void_p:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _dev(t, dtype=None, name="tensor"):
    """Device pointer of a torch tensor after checking device / dtype / inner contiguity."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU (no CPU path exists)")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name}: dtype {t.dtype}, expected {dtype}")
    if t.dim() > 0 and t.numel() > 0 and t.stride(-1) != 1:
        raise ValueError(f"{name}: innermost axis must be contiguous")
    return t.data_ptr()


def set_option(name: str, value: int) -> None:
    _check(lib().dlm_set_option(name.encode(), int(value)))


def kv_seg(k=None, v=None, pos0: int = 0, rule: int = 0) -> KvSeg:
    """k, v: bf16 [B, Hkv, len, d] views (any batch/head/row strides) or None for an absent segment.
    rule: SEG_CAUSAL / SEG_EARLIER_BLOCKS / SEG_SAME_BLOCK (block-causal mask only)."""
    import torch
    s = KvSeg()
    s.rule = int(rule)
    if k is None or k.shape[2] == 0:
        s.k = s.v = None
        s.len = 0
        s.pos0 = int(pos0)
        return s
    if k.shape != v.shape or k.stride() != v.stride():
        raise ValueError("k and v of a segment must have the same shape and strides")
    s.k, s.v = _dev(k, torch.bfloat16, "k"), _dev(v, torch.bfloat16, "v")
    s.len, s.pos0 = int(k.shape[2]), int(pos0)
    s.stride_b, s.stride_h, s.stride_t = int(k.stride(0)), int(k.stride(1)), int(k.stride(2))
    return s


def block_attn_workspace_bytes(q, prefix: Optional[Tuple] = None, block: Optional[Tuple] = None,
                               suffix: Optional[Tuple] = None, **kw) -> int:
    """Bytes of workspace dlm_block_attn wants for this call (0 for most shapes)."""
    kw.pop("workspace", None)
    kw.pop("stream", None)
    a = _attn_args(q, q, prefix, block, suffix, **kw)
    return int(lib().dlm_block_attn_workspace_bytes(C.byref(a)))


def block_attn(q, out, prefix: Optional[Tuple] = None, block: Optional[Tuple] = None,
               suffix: Optional[Tuple] = None, *, stream=None, **kw) -> None:
    """q, out: bf16 [B, Lq, Hq, d]; each segment is (k, v, pos0[, rule]) with k, v bf16 [B, Hkv, len, d].
    Keywords: n_kv_heads, mask_mode, block_size, q_pos0, scale, prefix_len_b, lse, workspace (a uint8 tensor of
    block_attn_workspace_bytes(...) bytes when that is not 0), seq_active (optional int32 [B] on the device;
    sequences with a 0 are skipped: out / lse rows untouched)."""
    a = _attn_args(q, out, prefix, block, suffix, **kw)
    _check(lib().dlm_block_attn(C.byref(a), _stream(stream)))


def _attn_args(q, out, prefix, block, suffix, *, n_kv_heads: Optional[int] = None,
               mask_mode: int = MASK_FULL, block_size: int = 0, q_pos0: int = 0, scale: float = 0.0,
               prefix_len_b=None, lse=None, workspace=None, seq_active=None) -> AttnArgs:
    import torch
    a = AttnArgs()
    a.struct_size = C.sizeof(AttnArgs)
    B, Lq, Hq, d = q.shape
    if out.shape != q.shape:
        raise ValueError("out must have q's shape")
    segs = [prefix, block, suffix]
    hkv = n_kv_heads
    for sg in segs:
        if sg is not None and sg[0] is not None:
            hkv = sg[0].shape[1]
    a.B, a.Lq, a.Hq, a.Hkv, a.d = B, Lq, Hq, int(hkv if hkv else Hq), d
    a.q = _dev(q, torch.bfloat16, "q")
    a.q_stride_b, a.q_stride_t, a.q_stride_h = q.stride(0), q.stride(1), q.stride(2)
    a.prefix = kv_seg(*prefix) if prefix else kv_seg()
    a.block = kv_seg(*block) if block else kv_seg()
    a.suffix = kv_seg(*suffix) if suffix else kv_seg()
    a.prefix_len_b = _dev(prefix_len_b, torch.int32, "prefix_len_b")
    a.mask_mode, a.block_size, a.q_pos0, a.scale = int(mask_mode), int(block_size), int(q_pos0), float(scale)
    a.out = _dev(out, torch.bfloat16, "out")
    a.o_stride_b, a.o_stride_t, a.o_stride_h = out.stride(0), out.stride(1), out.stride(2)
    if lse is not None and (not lse.is_contiguous() or tuple(lse.shape) != (B, Hq, Lq)):
        raise ValueError("lse must be contiguous fp32 [B, Hq, Lq]")
    a.lse = _dev(lse, torch.float32, "lse")
    a.workspace = _dev(workspace, None, "workspace")
    a.workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    if seq_active is not None:
        if seq_active.numel() != B or not seq_active.is_contiguous():
            raise ValueError("seq_active must be contiguous int32 [B]")
        a.seq_active = _dev(seq_active, torch.int32, "seq_active")
    return a


def varlen_attn(q, k, v, out, cu_seqlens, max_seqlen: int, *, mask_mode: int = MASK_FULL, block_size: int = 0,
                scale: float = 0.0, lse=None, stream=None) -> None:
    """Packed variable-length attention through dlm_block_attn: q, out bf16 [T, Hq, d]; k, v bf16 [T, Hkv, d];
    cu_seqlens int32 [B + 1] on the device; every sequence attends to itself only.  lse fp32 [Hq, T]."""
    import torch
    a = AttnArgs()
    a.struct_size = C.sizeof(AttnArgs)
    T, Hq, d = q.shape
    if out.shape != q.shape or k.shape != v.shape or k.stride() != v.stride() or k.shape[0] != T or k.shape[2] != d:
        raise ValueError("q/out [T, Hq, d] and k/v [T, Hkv, d] expected")
    B = cu_seqlens.numel() - 1
    a.B, a.Lq, a.Hq, a.Hkv, a.d = B, int(max_seqlen), Hq, k.shape[1], d
    a.q, a.q_stride_b, a.q_stride_t, a.q_stride_h = _dev(q, torch.bfloat16, "q"), 0, q.stride(0), q.stride(1)
    a.out, a.o_stride_b, a.o_stride_t, a.o_stride_h = _dev(out, torch.bfloat16, "out"), 0, out.stride(0), out.stride(1)
    a.prefix, a.suffix = kv_seg(), kv_seg()
    a.block.k, a.block.v = _dev(k, torch.bfloat16, "k"), _dev(v, torch.bfloat16, "v")
    a.block.len, a.block.pos0 = int(max_seqlen), 0
    a.block.stride_b, a.block.stride_t, a.block.stride_h = 0, k.stride(0), k.stride(1)
    a.mask_mode, a.block_size, a.q_pos0, a.scale = int(mask_mode), int(block_size), 0, float(scale)
    if lse is not None and (not lse.is_contiguous() or tuple(lse.shape) != (Hq, T)):
        raise ValueError("lse must be contiguous fp32 [Hq, T]")
    a.lse = _dev(lse, torch.float32, "lse")
    a.cu_seqlens, a.total_tokens = _dev(cu_seqlens, torch.int32, "cu_seqlens"), T
    _check(lib().dlm_block_attn(C.byref(a), _stream(stream)))


def block_attn_bwd(q, out, d_out, lse, d_q, prefix: Optional[Tuple] = None, block: Optional[Tuple] = None,
                   suffix: Optional[Tuple] = None, *, d_prefix: Optional[Tuple] = None, d_block: Optional[Tuple] = None,
                   d_suffix: Optional[Tuple] = None, mask_mode: int = MASK_FULL, block_size: int = 0, q_pos0: int = 0,
                   scale: float = 0.0, cu_seqlens=None, max_seqlen: Optional[int] = None, workspace=None,
                   stream=None) -> None:
    """Gradients of block_attn.  Dense mode: q, out, d_out, d_q bf16 [B, Lq, Hq, d]; segments (k, v, pos0[, rule])
    with k, v [B, Hkv, len, d]; d_<segment> = (dk, dv) tensors with that segment's shape and strides, or None.
    Packed mode (cu_seqlens given): q, out, d_out, d_q [T, Hq, d]; block = (k, v) with k, v [T, Hkv, d]."""
    import torch
    a = AttnBwdArgs()
    a.struct_size = C.sizeof(AttnBwdArgs)
    packed = cu_seqlens is not None
    if packed:
        T, Hq, d = q.shape
        B, Lq = cu_seqlens.numel() - 1, int(max_seqlen)
        sb = lambda t: (0, t.stride(0), t.stride(1))
    else:
        B, Lq, Hq, d = q.shape
        sb = lambda t: (t.stride(0), t.stride(1), t.stride(2))
    for t, name in ((out, "out"), (d_out, "d_out")) + (((d_q, "d_q"),) if d_q is not None else ()):
        if t.shape != q.shape:
            raise ValueError(f"{name} must have q's shape")
    a.q, (a.q_stride_b, a.q_stride_t, a.q_stride_h) = _dev(q, torch.bfloat16, "q"), sb(q)
    a.out, (a.o_stride_b, a.o_stride_t, a.o_stride_h) = _dev(out, torch.bfloat16, "out"), sb(out)
    a.d_out, (a.do_stride_b, a.do_stride_t, a.do_stride_h) = _dev(d_out, torch.bfloat16, "d_out"), sb(d_out)
    if d_q is not None:
        a.d_q, (a.dq_stride_b, a.dq_stride_t, a.dq_stride_h) = _dev(d_q, torch.bfloat16, "d_q"), sb(d_q)
    if not lse.is_contiguous():
        raise ValueError("lse must be contiguous")
    a.lse = _dev(lse, torch.float32, "lse")
    hkv = Hq
    if packed:
        k, v = block[0], block[1]
        if k.shape != v.shape or k.stride() != v.stride():
            raise ValueError("k and v must share shape and strides")
        hkv = k.shape[1]
        a.prefix, a.suffix = kv_seg(), kv_seg()
        a.block.k, a.block.v = _dev(k, torch.bfloat16, "k"), _dev(v, torch.bfloat16, "v")
        a.block.len, a.block.pos0, a.block.rule = Lq, 0, int(block[3]) if len(block) > 3 else 0
        a.block.stride_b, a.block.stride_t, a.block.stride_h = 0, k.stride(0), k.stride(1)
        a.cu_seqlens, a.total_tokens = _dev(cu_seqlens, torch.int32, "cu_seqlens"), T
    else:
        for sg in (prefix, block, suffix):
            if sg is not None and sg[0] is not None:
                hkv = sg[0].shape[1]
        a.prefix = kv_seg(*prefix) if prefix else kv_seg()
        a.block = kv_seg(*block) if block else kv_seg()
        a.suffix = kv_seg(*suffix) if suffix else kv_seg()
    a.B, a.Lq, a.Hq, a.Hkv, a.d = B, Lq, Hq, hkv, d
    for name, grads, seg in (("prefix", d_prefix, prefix), ("block", d_block, block), ("suffix", d_suffix, suffix)):
        if grads is None:
            continue
        dk, dv = grads
        if seg is None or dk.shape != seg[0].shape or dk.stride() != seg[0].stride() or dv.stride() != seg[0].stride():
            raise ValueError(f"d_{name} must match the {name} segment's shape and strides")
        setattr(a, f"d_{name}_k", _dev(dk, torch.bfloat16, "dk"))
        setattr(a, f"d_{name}_v", _dev(dv, torch.bfloat16, "dv"))
    a.mask_mode, a.block_size, a.q_pos0, a.scale = int(mask_mode), int(block_size), int(q_pos0), float(scale)
    need = int(lib().dlm_block_attn_bwd_workspace_bytes(C.byref(a)))
    if workspace is None:
        raise ValueError(f"workspace of {need} bytes required")
    a.workspace = _dev(workspace, None, "workspace")
    a.workspace_bytes = workspace.numel() * workspace.element_size()
    _check(lib().dlm_block_attn_bwd(C.byref(a), _stream(stream)))


def block_attn_bwd_workspace_bytes(n_rows: int, Hq: int) -> int:
    """n_rows = B * Lq (dense) or the total token count (packed)."""
    return int(n_rows) * int(Hq) * 4


def lmhead_workspace_bytes(M: int, V: int, sample: bool = False, conf_mode: int = CONF_TOKEN_PROB) -> int:
    a = LmheadArgs()
    a.struct_size = C.sizeof(LmheadArgs)
    a.M, a.V, a.Dh = int(M), int(V), 64
    a.sample, a.conf_mode = int(bool(sample)), int(conf_mode)
    return int(lib().dlm_lmhead_workspace_bytes(C.byref(a)))


def lmhead_confidence(hidden, w, conf, tok, *, stream=None, static_scratch: bool = False, **kw) -> None:
    """hidden bf16 [rows, Dh]; w bf16 [V, Dh]; conf fp32 / tok int32 outputs.  Keywords: M, row_idx, m_dev,
    inv_temperature, forbid_token, out_scatter, lse, zmax, z2nd, target, ztarget, workspace (a uint8 tensor),
    sample_seed (None = arg-max token; an integer = Gumbel-max sample with that seed), sample_step, sample_stream,
    conf_mode, M_expected (a guess of the row count m_dev holds, 0 = none; only the choice of kernel shape depends on it).
    static_scratch: call dlm_lmhead_confidence_static (the library's built-in scratch; no workspace tensor)."""
    a = _lmhead_args(hidden, w, conf, tok, **kw)
    fn = lib().dlm_lmhead_confidence_static if static_scratch else lib().dlm_lmhead_confidence
    _check(fn(C.byref(a), _stream(stream)))


def _lmhead_args(hidden, w, conf, tok, *, M: Optional[int] = None, row_idx=None, m_dev=None,
                 inv_temperature: float = 1.0, forbid_token: int = -1, out_scatter: bool = False,
                 lse=None, zmax=None, z2nd=None, target=None, ztarget=None, workspace=None,
                 sample_seed: Optional[int] = None, sample_step: int = 0, sample_stream: int = 0,
                 conf_mode: int = CONF_TOKEN_PROB, M_expected: int = 0) -> LmheadArgs:
    import torch
    a = LmheadArgs()
    a.struct_size = C.sizeof(LmheadArgs)
    rows, Dh = hidden.shape
    V = w.shape[0]
    if w.shape[1] != Dh:
        raise ValueError("w must be [V, Dh]")
    if M is None:
        M = row_idx.shape[0] if row_idx is not None else rows
    a.M, a.Dh, a.V = int(M), int(Dh), int(V)
    a.hidden, a.hidden_stride_row = _dev(hidden, torch.bfloat16, "hidden"), hidden.stride(0)
    a.row_idx = _dev(row_idx, torch.int32, "row_idx")
    a.m_dev = _dev(m_dev, torch.int32, "m_dev")
    a.w, a.w_stride_row = _dev(w, torch.bfloat16, "w"), w.stride(0)
    a.inv_temperature, a.forbid_token, a.out_scatter = float(inv_temperature), int(forbid_token), int(bool(out_scatter))
    a.conf, a.tok = _dev(conf, torch.float32, "conf"), _dev(tok, torch.int32, "tok")
    a.lse, a.zmax, a.z2nd = (_dev(lse, torch.float32, "lse"), _dev(zmax, torch.float32, "zmax"),
                             _dev(z2nd, torch.float32, "z2nd"))
    a.target, a.ztarget = _dev(target, torch.int32, "target"), _dev(ztarget, torch.float32, "ztarget")
    a.workspace = _dev(workspace, None, "workspace")
    a.workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    a.conf_mode = int(conf_mode)
    a.M_expected = int(M_expected)
    if sample_seed is not None:
        a.sample, a.sample_seed = 1, int(sample_seed) & 0xFFFFFFFFFFFFFFFF
        a.sample_step, a.sample_stream = int(sample_step) & 0xFFFFFFFF, int(sample_stream) & 0xFFFFFFFF
    return a


def unmask_commit(conf, tok, x, mask, n_commit, remaining, *, stream=None, **kw) -> None:
    """conf fp32 / tok int32 dense [B, n_pos]; x int32 [B, L]; mask uint8 [B, n_pos] (row-strided views are fine).
    Keywords: x_pos0 (required), group_len, rule, threshold, force_top1, k, commit_now, next_row_idx, next_m, commit_step,
    step, writeback, src_block, cache_k, cache_v, cache_pos0, active_in, host_remaining_total / host_remaining_max (optional
    pinned CPU int32 tensors of 1 element each that the kernel writes through)."""
    a = _commit_args(conf, tok, x, mask, n_commit, remaining, **kw)
    _check(lib().dlm_unmask_commit(C.byref(a), _stream(stream)))


def _commit_args(conf, tok, x, mask, n_commit, remaining, *, x_pos0: int, group_len: Optional[int] = None,
                 rule: int = RULE_THRESHOLD, threshold: float = 0.0, force_top1: bool = True, k: int = 0,
                 commit_now=None, next_row_idx=None, next_m=None, commit_step=None, step: int = 0,
                 writeback: int = WB_NONE, src_block: Optional[Tuple] = None, cache_k=None, cache_v=None,
                 cache_pos0: int = 0, host_remaining_total=None, active_in=None, host_remaining_max=None) -> CommitArgs:
    import torch
    a = CommitArgs()
    a.struct_size = C.sizeof(CommitArgs)
    B, n_pos = mask.shape
    if not conf.is_contiguous() or not tok.is_contiguous() or conf.numel() != B * n_pos or tok.numel() != B * n_pos:
        raise ValueError("conf / tok must be contiguous [B, n_pos]")
    a.B, a.n_pos, a.group_len = B, n_pos, int(n_pos if group_len is None else group_len)
    a.rule, a.threshold, a.force_top1, a.k = int(rule), float(threshold), int(bool(force_top1)), int(k)
    a.conf, a.tok = _dev(conf, torch.float32, "conf"), _dev(tok, torch.int32, "tok")
    a.x, a.x_stride_b, a.x_pos0 = _dev(x, torch.int32, "x"), x.stride(0), int(x_pos0)
    a.mask, a.mask_stride_b = _dev(mask, torch.uint8, "mask"), mask.stride(0)
    for name, t in (("commit_now", commit_now), ("commit_step", commit_step)):
        if t is not None and (not t.is_contiguous() or t.numel() != B * n_pos):
            raise ValueError(f"{name} must be contiguous [B, n_pos]")
    a.commit_now = _dev(commit_now, torch.uint8, "commit_now")
    a.n_commit, a.remaining = _dev(n_commit, torch.int32, "n_commit"), _dev(remaining, torch.int32, "remaining")
    a.next_row_idx, a.next_m = _dev(next_row_idx, torch.int32, "next_row_idx"), _dev(next_m, torch.int32, "next_m")
    a.commit_step, a.step = _dev(commit_step, torch.int16, "commit_step"), int(step)
    a.writeback = int(writeback)
    if writeback != WB_NONE:
        a.src_block = kv_seg(*src_block)
        if cache_k.stride() != cache_v.stride():
            raise ValueError("cache_k and cache_v must share strides")
        a.cache_k, a.cache_v = _dev(cache_k, torch.bfloat16, "cache_k"), _dev(cache_v, torch.bfloat16, "cache_v")
        a.c_stride_b, a.c_stride_h, a.c_stride_t = cache_k.stride(0), cache_k.stride(1), cache_k.stride(2)
        a.cache_pos0, a.Hkv, a.d = int(cache_pos0), int(cache_k.shape[1]), int(cache_k.shape[3])
        if active_in is not None:
            if active_in.numel() != B or not active_in.is_contiguous():
                raise ValueError("active_in must be contiguous [B]")
            a.active_in = _dev(active_in, torch.int32, "active_in")
    if host_remaining_total is not None:
        if host_remaining_total.is_cuda or not host_remaining_total.is_pinned() or host_remaining_total.dtype != torch.int32:
            raise ValueError("host_remaining_total must be a pinned CPU int32 tensor")
        a.host_remaining_total = host_remaining_total.data_ptr()
    if host_remaining_max is not None:
        if host_remaining_max.is_cuda or not host_remaining_max.is_pinned() or host_remaining_max.dtype != torch.int32:
            raise ValueError("host_remaining_max must be a pinned CPU int32 tensor")
        a.host_remaining_max = host_remaining_max.data_ptr()
    return a


def mask_compact(mask, row_idx, m_out, stream=None) -> None:
    import torch
    B, n_pos = mask.shape
    _check(lib().dlm_mask_compact(_dev(mask, torch.uint8, "mask"), mask.stride(0), B, n_pos,
                                  _dev(row_idx, torch.int32, "row_idx"), _dev(m_out, torch.int32, "m_out"),
                                  _stream(stream)))


def kv_refresh(src_k, src_v, cache_k, cache_v, cache_pos0: int, stream=None) -> None:
    """Copy src K,V [B, Hkv, len, d] into cache rows [cache_pos0, cache_pos0 + len)."""
    import torch
    seg = kv_seg(src_k, src_v, 0)
    if cache_k.stride() != cache_v.stride():
        raise ValueError("cache_k and cache_v must share strides")
    B, Hkv, _, d = src_k.shape
    if cache_pos0 + src_k.shape[2] > cache_k.shape[2]:
        raise ValueError("refresh would write past the end of the cache")
    _check(lib().dlm_kv_refresh(C.byref(seg), B, Hkv, d, _dev(cache_k, torch.bfloat16, "cache_k"),
                                _dev(cache_v, torch.bfloat16, "cache_v"), cache_k.stride(0), cache_k.stride(1),
                                cache_k.stride(2), int(cache_pos0), _stream(stream)))


def seq_logprob(ztarget, lse, mask, out, *, weight=None, n_terms=None, stream=None) -> None:
    """out[b] = weight[b] * sum over masked positions of (ztarget - lse); ztarget, lse fp32 [B, n_pos]."""
    import torch
    B, n_pos = mask.shape
    if not ztarget.is_contiguous() or not lse.is_contiguous() or ztarget.numel() != B * n_pos or lse.numel() != B * n_pos:
        raise ValueError("ztarget / lse must be contiguous [B, n_pos]")
    _check(lib().dlm_seq_logprob(_dev(ztarget, torch.float32, "ztarget"), _dev(lse, torch.float32, "lse"),
                                 _dev(mask, torch.uint8, "mask"), mask.stride(0), _dev(weight, torch.float32, "weight"),
                                 B, n_pos, _dev(out, torch.float32, "out"), _dev(n_terms, torch.int32, "n_terms"),
                                 _stream(stream)))
