"""CPU-only checks of the boundary: the library loads, exports every symbol the
header declares, and turns bad arguments into error codes before any launch."""
import ctypes
import os
import re

import pytest

import paper_2512_02337_amd as specpv
from paper_2512_02337_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "specpv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(specpv_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = specpv.load()
    names = _declared()
    assert set(names) == set(specpv.EXPORTS), names
    for n in names:
        assert getattr(lib, n) is not None
    assert specpv.specpv_version() >= 100
    assert "workspace" in specpv.specpv_strerror(-2)


def _kv(**over):
    d = dict(k=0x1000, v=0x2000, stride_b=1 << 20, stride_h=1 << 14, stride_t=128, ctx_len=0x3000,
             batch=1, n_kv_heads=8, head_dim=128, block_size=64, max_blocks=16, dtype=1)
    d.update(over)
    return binding._KV(**d)


def _tree(**over):
    d = dict(q=0x4000, kd=0x5000, vd=0x6000, parent=0x7000, M=60, n_q_heads=32, last_node=0)
    d.update(over)
    return binding._Tree(**d)


def _cfg(**over):
    d = dict(n_sink_blocks=1, n_recent_blocks=2, k_blocks=4, reduce=0)
    d.update(over)
    return binding._Cfg(**d)


def test_bad_arguments_are_rejected_on_the_host():
    """Pointers are fake but never dereferenced: every case must fail validation
    before anything is launched (this runs without a GPU)."""
    lib = specpv.load()
    B = ctypes.byref
    vp = ctypes.c_void_p
    ws_bytes = lib.specpv_workspace_bytes(B(_kv()), B(_tree()), B(_cfg()))
    assert ws_bytes > 0
    # descriptors
    assert lib.specpv_workspace_bytes(B(_kv(head_dim=96)), B(_tree()), B(_cfg())) == 0
    assert lib.specpv_block_summarize(None, 0, -1, vp(16), vp(32), None) == -1
    assert lib.specpv_block_summarize(B(_kv(k=None)), 0, -1, vp(16), vp(32), None) == -1
    assert lib.specpv_block_summarize(B(_kv(head_dim=96)), 0, -1, vp(16), vp(32), None) == -1
    assert lib.specpv_block_summarize(B(_kv(dtype=5)), 0, -1, vp(16), vp(32), None) == -1
    assert lib.specpv_block_summarize(B(_kv(stride_t=64)), 0, -1, vp(16), vp(32), None) == -1
    assert lib.specpv_block_summarize(B(_kv(stride_t=132)), 0, -1, vp(16), vp(32), None) == -1
    assert lib.specpv_block_summarize(B(_kv(k=0x1004)), 0, -1, vp(16), vp(32), None) == -1
    assert lib.specpv_block_summarize(B(_kv()), 0, -1, None, vp(32), None) == -1
    assert lib.specpv_block_summarize(B(_kv()), -3, -1, vp(16), vp(32), None) == -1
    # tree limits
    args = (vp(0x100), vp(0x200), 7, vp(0x300), None, vp(0x8000), ws_bytes, None)
    assert lib.specpv_partial_verify_attn(B(_kv()), B(_tree(M=129)), *args) == -3
    assert lib.specpv_partial_verify_attn(B(_kv()), B(_tree(M=0)), *args) == -1
    assert lib.specpv_partial_verify_attn(B(_kv()), B(_tree(n_q_heads=30)), *args) == -1
    assert lib.specpv_partial_verify_attn(B(_kv(n_kv_heads=1)), B(_tree(n_q_heads=32)), *args) == -3
    assert lib.specpv_partial_verify_attn(B(_kv()), B(_tree(kd=None)), *args) == -1
    assert lib.specpv_partial_verify_attn(B(_kv()), B(_tree(parent=None)), *args) == -1
    # workspace
    assert lib.specpv_partial_verify_attn(B(_kv()), B(_tree()), vp(0x100), vp(0x200), 7, vp(0x300), None,
                                          vp(0x8000), 16, None) == -2
    assert lib.specpv_partial_verify_attn(B(_kv()), B(_tree()), vp(0x100), vp(0x200), 7, vp(0x300), None,
                                          None, ws_bytes, None) == -2
    assert lib.specpv_partial_verify_attn(B(_kv()), B(_tree()), vp(0x100), None, 7, vp(0x300), None,
                                          vp(0x8000), ws_bytes, None) == -1
    # selection config
    sel = (vp(0x100), vp(0x200), None, vp(0x8000), ws_bytes, None)
    assert lib.specpv_select_blocks(B(_kv()), B(_tree()), vp(16), vp(32), B(_cfg(k_blocks=-1)), *sel) == -1
    assert lib.specpv_select_blocks(B(_kv()), B(_tree()), vp(16), vp(32), B(_cfg(reduce=9)), *sel) == -1
    assert lib.specpv_select_blocks(B(_kv()), B(_tree(last_node=60)), vp(16), vp(32), B(_cfg(reduce=2)), *sel) == -1
    assert lib.specpv_select_blocks(B(_kv()), B(_tree()), vp(16), vp(32), None, *sel) == -1
    assert lib.specpv_select_blocks(B(_kv()), B(_tree()), vp(16), vp(32), B(_cfg()), vp(0x100), vp(0x200), None,
                                    None, 0, None) == -2
    assert lib.specpv_full_verify_refresh(B(_kv()), B(_tree()), vp(16), vp(32), 0, B(_cfg()), None, None,
                                          vp(0x100), vp(0x200), None, vp(0x8000), ws_bytes, None) == -1


def test_binding_refuses_cpu_tensors():
    import torch
    k = torch.zeros((1, 1, 64, 64))
    with pytest.raises(ValueError):
        specpv.KV(k, k, torch.zeros((1,), dtype=torch.int32), 16)
