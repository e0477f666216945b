"""The C ABI without a GPU: every declared symbol is exported, the ctypes structs
match the header's layout, and argument validation rejects bad calls before any
device work.  No compute call is made here."""
import ctypes as C
import os
import re
import subprocess
import sys

import pytest

from paper_2604_04215_amd import binding as dlm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "dlm.h")


def _declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(dlm_[a-z_0-9]+)\s*\(", src)))


def test_every_declared_symbol_is_exported():
    names = _declared_functions()
    assert set(names) == set(dlm.EXPORTS)
    L = dlm.lib()
    for n in names:
        assert getattr(L, n) is not None
    assert L.dlm_version() >= 100


def test_struct_layout_matches_header(tmp_path):
    prog = tmp_path / "layout.c"
    prog.write_text(r'''
#include <stdio.h>
#include <stddef.h>
#include "dlm.h"
int main(void) {
  printf("%zu %zu %zu %zu\n", sizeof(dlm_kv_seg), sizeof(dlm_attn_args), sizeof(dlm_lmhead_args), sizeof(dlm_commit_args));
  printf("%zu %zu %zu %zu\n", offsetof(dlm_attn_args, suffix), offsetof(dlm_attn_args, scale), offsetof(dlm_attn_args, lse), offsetof(dlm_attn_args, total_tokens));
  printf("%zu %zu %zu %zu\n", offsetof(dlm_lmhead_args, w), offsetof(dlm_lmhead_args, forbid_token), offsetof(dlm_lmhead_args, conf), offsetof(dlm_lmhead_args, workspace));
  printf("%zu %zu %zu %zu\n", offsetof(dlm_commit_args, conf), offsetof(dlm_commit_args, x_pos0), offsetof(dlm_commit_args, src_block), offsetof(dlm_commit_args, d));
  printf("%zu %zu %zu %zu\n", offsetof(dlm_attn_args, seq_active), offsetof(dlm_lmhead_args, M_expected), offsetof(dlm_commit_args, host_remaining_total), offsetof(dlm_commit_args, active_in));
  return 0;
}''')
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-std=c11", "-I", os.path.join(ROOT, "include"), str(prog), "-o", str(exe)])
    got = [[int(t) for t in line.split()] for line in subprocess.check_output([str(exe)], text=True).splitlines()]
    A, Lm, Cm = dlm.AttnArgs, dlm.LmheadArgs, dlm.CommitArgs
    want = [[C.sizeof(dlm.KvSeg), C.sizeof(A), C.sizeof(Lm), C.sizeof(Cm)],
            [A.suffix.offset, A.scale.offset, A.lse.offset, A.total_tokens.offset],
            [Lm.w.offset, Lm.forbid_token.offset, Lm.conf.offset, Lm.workspace.offset],
            [Cm.conf.offset, Cm.x_pos0.offset, Cm.src_block.offset, Cm.d.offset],
            [A.seq_active.offset, Lm.M_expected.offset, Cm.host_remaining_total.offset, Cm.active_in.offset]]
    assert got == want


def _attn(**kw):
    a = dlm.AttnArgs()
    a.struct_size = C.sizeof(dlm.AttnArgs)
    a.B, a.Lq, a.Hq, a.Hkv, a.d = 1, 4, 4, 2, 128
    a.q = a.out = 0x1000
    a.q_stride_b = a.o_stride_b = 4 * 4 * 128
    a.q_stride_t = a.o_stride_t = 4 * 128
    a.q_stride_h = a.o_stride_h = 128
    for k, v in kw.items():
        setattr(a, k, v)
    return a


def test_attn_validation():
    L = dlm.lib()
    assert L.dlm_block_attn(None, None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_block_attn(C.byref(_attn(struct_size=8)), None) == dlm.DLM_ERR_INVALID_ARG
    assert "struct_size" in dlm.last_error()
    assert L.dlm_block_attn(C.byref(_attn(Hkv=3)), None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_block_attn(C.byref(_attn(d=96)), None) == dlm.DLM_ERR_UNSUPPORTED
    assert "head_dim" in dlm.last_error()
    assert L.dlm_block_attn(C.byref(_attn(mask_mode=7)), None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_block_attn(C.byref(_attn(mask_mode=dlm.MASK_BLOCK_CAUSAL, block_size=0)), None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_block_attn(C.byref(_attn(q=0x1004)), None) == dlm.DLM_ERR_UNSUPPORTED      # misaligned
    assert L.dlm_block_attn(C.byref(_attn(q_stride_t=4 * 128 + 4)), None) == dlm.DLM_ERR_UNSUPPORTED
    assert L.dlm_block_attn(C.byref(_attn(q=None)), None) == dlm.DLM_ERR_INVALID_ARG
    bad = _attn()
    bad.prefix.len = 5                       # segment with null pointers
    assert L.dlm_block_attn(C.byref(bad), None) == dlm.DLM_ERR_INVALID_ARG
    bad.prefix.len = -1
    assert L.dlm_block_attn(C.byref(bad), None) == dlm.DLM_ERR_INVALID_ARG
    bad = _attn()
    bad.block.rule = 3
    assert L.dlm_block_attn(C.byref(bad), None) == dlm.DLM_ERR_INVALID_ARG
    bad.block.rule = dlm.SEG_SAME_BLOCK       # a segment rule without the block-causal mask
    assert L.dlm_block_attn(C.byref(bad), None) == dlm.DLM_ERR_INVALID_ARG
    # empty problems are fine and do nothing
    assert L.dlm_block_attn(C.byref(_attn(B=0)), None) == dlm.DLM_OK
    assert L.dlm_block_attn(C.byref(_attn(Lq=0)), None) == dlm.DLM_OK
    assert L.dlm_block_attn_workspace_bytes(C.byref(_attn())) == 0
    # packed variable-length mode: block segment only, block.len == Lq, token count within B * Lq
    def packed(**kw):
        a = _attn(cu_seqlens=0x2000, total_tokens=4)
        a.block.k = a.block.v = 0x3000
        a.block.len, a.block.stride_t, a.block.stride_h = 4, 2 * 128, 128
        for k, v in kw.items():
            setattr(a, k, v)
        return a
    a = packed()
    a.prefix.k = a.prefix.v = 0x3000
    a.prefix.len, a.prefix.stride_t = 8, 128
    assert L.dlm_block_attn(C.byref(a), None) == dlm.DLM_ERR_INVALID_ARG
    assert "packed" in dlm.last_error()
    assert L.dlm_block_attn(C.byref(packed(prefix_len_b=0x4000)), None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_block_attn(C.byref(packed(Lq=8)), None) == dlm.DLM_ERR_INVALID_ARG          # block.len != Lq
    assert L.dlm_block_attn(C.byref(packed(total_tokens=5)), None) == dlm.DLM_ERR_INVALID_ARG    # > B * Lq
    assert L.dlm_block_attn(C.byref(packed(total_tokens=-1)), None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_block_attn(C.byref(packed(B=0, total_tokens=0)), None) == dlm.DLM_OK
    assert L.dlm_seq_logprob(None, None, None, 0, None, 2, 4, None, None, None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_seq_logprob(None, None, None, 0, None, 0, 4, None, None, None) == dlm.DLM_OK
    assert L.dlm_seq_logprob(0x1000, 0x1000, 0x1000, 2, None, 2, 4, 0x1000, None, None) == dlm.DLM_ERR_INVALID_ARG


def _lm(**kw):
    a = dlm.LmheadArgs()
    a.struct_size = C.sizeof(dlm.LmheadArgs)
    a.M, a.Dh, a.V = 8, 256, 1000
    a.hidden = a.w = a.conf = a.tok = 0x1000
    a.hidden_stride_row = a.w_stride_row = 256
    a.inv_temperature, a.forbid_token = 1.0, -1
    for k, v in kw.items():
        setattr(a, k, v)
    return a


def test_lmhead_validation():
    L = dlm.lib()
    assert L.dlm_lmhead_confidence(None, None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_lmhead_confidence(C.byref(_lm(struct_size=1)), None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_lmhead_confidence(C.byref(_lm(Dh=100, hidden_stride_row=104, w_stride_row=104)), None) == dlm.DLM_ERR_UNSUPPORTED
    assert L.dlm_lmhead_confidence(C.byref(_lm(V=0)), None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_lmhead_confidence(C.byref(_lm(forbid_token=1000)), None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_lmhead_confidence(C.byref(_lm(inv_temperature=0.0)), None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_lmhead_confidence(C.byref(_lm(target=0x1000)), None) == dlm.DLM_ERR_INVALID_ARG   # no ztarget
    assert L.dlm_lmhead_confidence(C.byref(_lm(conf=None)), None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_lmhead_confidence(C.byref(_lm(w_stride_row=128)), None) == dlm.DLM_ERR_INVALID_ARG
    need = L.dlm_lmhead_workspace_bytes(C.byref(_lm()))
    assert need >= 8 * 16 * (1000 // 256)
    assert L.dlm_lmhead_confidence(C.byref(_lm()), None) == dlm.DLM_ERR_WORKSPACE                 # none given
    assert L.dlm_lmhead_confidence(C.byref(_lm(workspace=0x2000, workspace_bytes=need - 1)), None) == dlm.DLM_ERR_WORKSPACE
    assert "workspace" in dlm.last_error()
    assert L.dlm_lmhead_confidence(C.byref(_lm(M=0)), None) == dlm.DLM_OK
    assert dlm.lmhead_workspace_bytes(0, 1000) == 0
    assert dlm.lmhead_workspace_bytes(256, 126464) >= 256 * 16 * (126464 // 256)


def _cm(**kw):
    a = dlm.CommitArgs()
    a.struct_size = C.sizeof(dlm.CommitArgs)
    a.B, a.n_pos, a.group_len = 2, 32, 32
    a.rule, a.threshold, a.force_top1, a.k = dlm.RULE_THRESHOLD, 0.9, 1, 0
    a.conf = a.tok = a.x = a.mask = a.n_commit = a.remaining = 0x1000
    a.x_stride_b, a.x_pos0, a.mask_stride_b = 64, 16, 32
    for k, v in kw.items():
        setattr(a, k, v)
    return a


def test_commit_validation():
    L = dlm.lib()
    assert L.dlm_unmask_commit(None, None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_unmask_commit(C.byref(_cm(struct_size=4)), None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_unmask_commit(C.byref(_cm(group_len=0)), None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_unmask_commit(C.byref(_cm(group_len=5)), None) == dlm.DLM_ERR_INVALID_ARG       # 32 % 5
    assert L.dlm_unmask_commit(C.byref(_cm(group_len=2048, n_pos=2048, x_stride_b=4096, mask_stride_b=2048)), None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_unmask_commit(C.byref(_cm(rule=5)), None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_unmask_commit(C.byref(_cm(rule=dlm.RULE_TOPK, k=0)), None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_unmask_commit(C.byref(_cm(threshold=float("nan"))), None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_unmask_commit(C.byref(_cm(x_stride_b=40)), None) == dlm.DLM_ERR_INVALID_ARG     # 16 + 32 > 40
    assert L.dlm_unmask_commit(C.byref(_cm(mask=None)), None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_unmask_commit(C.byref(_cm(next_m=0x1000)), None) == dlm.DLM_ERR_INVALID_ARG     # without next_row_idx
    assert L.dlm_unmask_commit(C.byref(_cm(writeback=9)), None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_unmask_commit(C.byref(_cm(writeback=dlm.WB_BLOCK_WHEN_DONE, Hkv=2, d=128)), None) == dlm.DLM_ERR_INVALID_ARG  # null src
    def wb_active(**kw):   # a complete write-back request of the "while active" kind, then one thing wrong with it
        a = _cm(writeback=dlm.WB_WHILE_ACTIVE, Hkv=2, d=128, cache_k=0x2000, cache_v=0x3000, c_stride_b=65536,
                c_stride_h=8192, c_stride_t=128, n_commit=0x4000, remaining=0x5000, **kw)
        a.src_block.k, a.src_block.v, a.src_block.len = 0x6000, 0x7000, 32
        a.src_block.stride_b, a.src_block.stride_h, a.src_block.stride_t = 8192, 4096, 128
        return a
    assert L.dlm_unmask_commit(C.byref(wb_active()), None) == dlm.DLM_ERR_INVALID_ARG                    # no active_in
    assert L.dlm_unmask_commit(C.byref(wb_active(active_in=0x5000)), None) == dlm.DLM_ERR_INVALID_ARG   # aliases remaining
    assert L.dlm_unmask_commit(C.byref(wb_active(active_in=0x4000)), None) == dlm.DLM_ERR_INVALID_ARG   # aliases n_commit
    assert L.dlm_unmask_commit(C.byref(_cm(B=0)), None) == dlm.DLM_OK


def test_refresh_compact_option_validation():
    L = dlm.lib()
    seg = dlm.KvSeg()
    seg.len = 4
    assert L.dlm_kv_refresh(C.byref(seg), 1, 1, 128, None, None, 0, 0, 128, 0, None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_kv_refresh(C.byref(seg), 1, 1, 100, 0x1000, 0x1000, 0, 0, 128, 0, None) == dlm.DLM_ERR_UNSUPPORTED
    assert L.dlm_kv_refresh(None, 1, 1, 128, None, None, 0, 0, 128, 0, None) == dlm.DLM_ERR_INVALID_ARG
    seg.len = 0
    assert L.dlm_kv_refresh(C.byref(seg), 1, 1, 128, None, None, 0, 0, 128, 0, None) == dlm.DLM_OK
    assert L.dlm_mask_compact(None, 32, 2, 32, None, None, None) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_mask_compact(0x1000, 16, 2, 32, 0x1000, 0x1000, None) == dlm.DLM_ERR_INVALID_ARG   # stride < n_pos
    assert L.dlm_set_option(b"nope", 1) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_set_option(b"attn_variant", 99) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_set_option(b"attn_variant", 0) == dlm.DLM_OK
    assert L.dlm_set_option(b"attn_remap", 8) == dlm.DLM_ERR_INVALID_ARG
    assert L.dlm_set_option(b"attn_remap", 7) == dlm.DLM_OK


def test_binding_refuses_cpu_tensors():
    import torch
    q = torch.zeros((1, 4, 4, 128), dtype=torch.bfloat16)
    with pytest.raises(ValueError, match="GPU"):
        dlm.block_attn(q, q.clone())
    h = torch.zeros((4, 256), dtype=torch.bfloat16)
    with pytest.raises(ValueError, match="GPU"):
        dlm.lmhead_confidence(h, h, torch.zeros(4), torch.zeros(4, dtype=torch.int32))


def test_product_code_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2604_04215_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "liboracle" not in text, f
