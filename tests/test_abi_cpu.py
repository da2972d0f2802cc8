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
    d = dict(q=0x4000, kd=0x5000, vd=0x6000, parent=0x7000, M=60, n_q_heads=32, last_node=0, n_key_only=0)
    d.update(over)
    return binding._Tree(**d)


def _cfg(**over):
    d = dict(n_sink_blocks=1, n_recent_blocks=2, k_blocks=4, reduce=0, score=0, n_extra_slots=0)
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
    assert lib.specpv_partial_verify_attn(B(_kv()), B(_tree(n_key_only=-1)), *args) == -1
    assert lib.specpv_partial_verify_attn(B(_kv()), B(_tree(n_key_only=60)), *args) == -1   # no query node left
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
    assert lib.specpv_select_blocks(B(_kv()), B(_tree()), vp(16), vp(32), B(_cfg(score=2)), *sel) == -1
    assert lib.specpv_select_blocks(B(_kv()), B(_tree(last_node=60)), vp(16), vp(32), B(_cfg(reduce=2)), *sel) == -1
    assert lib.specpv_select_blocks(B(_kv()), B(_tree(last_node=3, n_key_only=4)), vp(16), vp(32), B(_cfg(reduce=2)), *sel) == -1
    assert lib.specpv_select_blocks(B(_kv()), B(_tree()), vp(16), vp(32), B(_cfg(n_extra_slots=-1)), *sel) == -1
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


def test_mode_policy_and_extended_parents_on_the_host():
    """Host-only entry points: the library's SelectMode and extended-tree parents against the
    hand-worked example and the oracle's own version (no GPU involved)."""
    import json
    import numpy as np
    import oracle
    import workloads
    g = json.load(open(os.path.join(ROOT, "tests", "golden", "mode_policy_hand_example.json")))
    names = {"FULL": specpv.MODE_FULL, "PARTIAL": specpv.MODE_PARTIAL, "REFRESH": specpv.MODE_REFRESH}
    for st in g["steps"]:
        got = specpv.specpv_select_mode(g["partial_budget_tokens"], g["pending_margin_tokens"], st["seq_len"],
                                        st["partial_ready"], st["n_pending"])
        assert got == names[st["mode"]], st
    for budget in (0, 7, 100):
        for margin in (0, 3):
            for seq_len in (0, 6, 7, 8, 100, 101, 5000):
                for ready in (False, True):
                    for pending in (0, 3, 4, 50):
                        assert specpv.specpv_select_mode(budget, margin, seq_len, ready, pending) == \
                            oracle.select_mode(seq_len, ready, pending, budget, margin)
    rng = np.random.default_rng(0)
    for n_pending in (0, 1, 20):
        for kind in ("uniform", "bounded", "chain", "star"):
            tree = workloads.make_tree(17, kind, rng).tolist()
            assert specpv.specpv_extend_parents(tree, n_pending) == oracle.extend_parents(tree, n_pending)
    lib = specpv.load()
    pol = binding._Policy(-1, 0)
    assert lib.specpv_select_mode(ctypes.byref(pol), 5, 0, 0) == -1
    assert lib.specpv_select_mode(None, 5, 0, 0) == -1
    bad = (ctypes.c_int32 * 3)(-1, 1, 0)     # parent[1] = 1 is not an earlier node
    out = (ctypes.c_int32 * 8)()
    assert lib.specpv_extend_parents(bad, 3, 2, out) == -1
    assert lib.specpv_extend_parents(bad, 3, 126, out) == -3
    # commit: fake pointers, never dereferenced
    vp = ctypes.c_void_p
    B = ctypes.byref
    ok_args = (vp(0x100), vp(0x200), 28, 60, vp(0x300), vp(0x400), vp(0x500), 8, 1, None, None, None, None,
               vp(0x8000), 1 << 17, None)
    assert lib.specpv_commit_accepted(None, *ok_args) == -1
    a = list(ok_args); a[0] = None
    assert lib.specpv_commit_accepted(B(_kv()), *a) == -1
    a = list(ok_args); a[8] = 7
    assert lib.specpv_commit_accepted(B(_kv()), *a) == -1          # unknown mode
    a = list(ok_args); a[2] = 125
    assert lib.specpv_commit_accepted(B(_kv()), *a) == -3          # buffer beyond the limits
    a = list(ok_args); a[14] = 2
    assert lib.specpv_commit_accepted(B(_kv()), *a) == -2          # workspace too small
    a = list(ok_args); a[11] = B(binding._Lists(0x900, None, 70))
    assert lib.specpv_commit_accepted(B(_kv()), *a) == -1          # lists without counts
    a = list(ok_args); a[11] = B(binding._Lists(0x900, 0xA00, 0))
    assert lib.specpv_commit_accepted(B(_kv()), *a) == -1          # empty list rows


def test_commit_of_all_layers_validates_on_the_host():
    """Fake pointers again: the layers of one call must share shape, strides, dtype and the length
    counters, and every table entry must be there."""
    lib = specpv.load()
    vp, P = ctypes.c_void_p, ctypes.POINTER

    def call(kvs, n=None, buf_k=(0x10000, 0x20000), buf_v=(0x30000, 0x40000), kmax=None, kmin=None, pending_cap=28):
        n = len(kvs) if n is None else n
        arr = (P(binding._KV) * len(kvs))(*[ctypes.pointer(k) for k in kvs])
        bk, bv = (vp * len(buf_k))(*buf_k), (vp * len(buf_v))(*buf_v)
        km = (vp * len(kmax))(*kmax) if kmax is not None else None
        kn = (vp * len(kmin))(*kmin) if kmin is not None else None
        return lib.specpv_commit_accepted_layers(arr, bk, bv, n, pending_cap, 60, vp(0x100), vp(0x200), vp(0x300), 8, 1,
                                                 km, kn, None, None, None, 0, None)
    two = [_kv(), _kv(k=0x9000, v=0xA000)]
    assert call(two) == -2                                    # everything valid up to the (missing) workspace
    assert call(two, n=0) == -1
    assert call(two, n=1000) == -1
    assert call([_kv(), _kv(ctx_len=0x3100)]) == -1           # two length arrays
    assert call([_kv(), _kv(max_blocks=32)]) == -1
    assert call([_kv(), _kv(stride_t=256)]) == -1
    assert call(two, buf_k=(0x10000, 0)) == -1
    assert call(two, buf_v=(0x30004, 0x40000)) == -1
    assert call(two, kmax=(0x50000, 0x60000)) == -1           # kmax without kmin
    assert call(two, kmax=(0x50000, 0), kmin=(0x70000, 0x80000)) == -1
    assert call(two, kmax=(0x50000, 0x60000), kmin=(0x70000, 0x80000)) == -2
    assert call(two, pending_cap=120) == -3


def test_workspace_size_is_a_consistent_split_plan():
    """specpv_workspace_bytes is host-only and deterministic.  Its value is the layout the calls use:
    64 KiB of arrival words + partial O [batch, Hq, splits + 1, M, D] fp32 + (m, l) pairs
    [batch, Hq, splits + 1, M, 2] fp32 + one score per block, each part rounded up to 256 bytes, for ONE
    split count between 1 and 64; and a selection can only add to what the full pass needs."""
    import random
    lib = specpv.load()
    up = lambda x: (x + 255) & ~255
    rnd = random.Random(5)

    def splits_of(total, batch, Hq, Hkv, M, D, nb):
        sc = up(batch * Hkv * nb * 4)
        for ns in range(1, 65):   # ns context splits + one slot for the draft-tree segment, behind 64 KiB of arrival words
            if 65536 + up(batch * Hq * (ns + 1) * M * D * 4) + up(batch * Hq * (ns + 1) * M * 8) + sc == total:
                return ns
        return None

    for _ in range(300):
        Hkv = rnd.choice([1, 2, 4, 8])
        G = rnd.choice([1, 2, 3, 4, 5, 8, 16])
        D = rnd.choice([64, 128])
        dtype = rnd.choice([0, 1])
        B = rnd.choice([7, 16, 32, 64, 128])
        nb = rnd.choice([1, 3, 17, 64, 500, 2048, 8192])
        M = rnd.choice([1, 9, 24, 60, 100, 128])
        batch = rnd.choice([1, 2, 4, 16])
        kv = _kv(batch=batch, n_kv_heads=Hkv, head_dim=D, block_size=B, max_blocks=nb, dtype=dtype,
                 stride_t=D, stride_h=nb * B * D, stride_b=Hkv * nb * B * D)
        tree = _tree(M=M, n_q_heads=Hkv * G)
        full = lib.specpv_workspace_bytes(ctypes.byref(kv), ctypes.byref(tree), None)
        assert full == lib.specpv_workspace_bytes(ctypes.byref(kv), ctypes.byref(tree), None)
        ns_full = splits_of(full, batch, Hkv * G, Hkv, M, D, nb)
        assert ns_full is not None, (Hkv, G, D, dtype, B, nb, M, batch, full)
        cfg = _cfg(n_sink_blocks=1, n_recent_blocks=2, k_blocks=rnd.choice([0, 4, 29, 61, 253]))
        both = lib.specpv_workspace_bytes(ctypes.byref(kv), ctypes.byref(tree), ctypes.byref(cfg))
        assert both >= full
        assert splits_of(both, batch, Hkv * G, Hkv, M, D, nb) is not None
    # no tree: only the per-sequence counters of the summary call
    assert lib.specpv_workspace_bytes(ctypes.byref(_kv()), None, None) >= 65536 + 4


def test_two_threads_may_call_at_once():
    """Host-only calls and host-side validation from two threads at the same time (fake pointers, nothing
    launched): the only state the library keeps is per-device set-up that is guarded for this."""
    import threading
    lib = specpv.load()
    B, vp = ctypes.byref, ctypes.c_void_p
    errs = []

    def work(seed):
        try:
            for i in range(300):
                kv, tree, cfg = _kv(max_blocks=16 + (i + seed) % 7), _tree(), _cfg()
                n = lib.specpv_workspace_bytes(B(kv), B(tree), B(cfg))
                assert n > 0 and n == lib.specpv_workspace_bytes(B(kv), B(tree), B(cfg))
                assert lib.specpv_partial_verify_attn(B(kv), B(tree), vp(0x100), vp(0x200), 7, vp(0x300), None,
                                                      vp(0x8000), 16, None) == -2
                assert lib.specpv_select_mode(B(binding._Policy(100, 3)), 500, 1, 4) == specpv.MODE_REFRESH
        except Exception as e:   # noqa: BLE001
            errs.append(e)
    ts = [threading.Thread(target=work, args=(s,)) for s in (0, 1)]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    assert not errs, errs
