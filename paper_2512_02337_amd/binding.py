"""ctypes binding of the C ABI in include/specpv.h (same names, same arguments).

The wrappers take torch tensors where the C call takes device pointers, check
dtype / device / contiguity (the C side cannot see those), and pass the current
torch stream.  They allocate nothing: outputs and workspace come from the caller.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libspecpv.so")

REDUCE_MEAN, REDUCE_MAX, REDUCE_LAST = 0, 1, 2
_REDUCE = {"mean": 0, "max": 1, "last": 2, 0: 0, 1: 1, 2: 2}
SCORE_EQ2, SCORE_CHANNEL_BOUND = 0, 1
_SCORE = {"eq2": 0, "channel_bound": 1, 0: 0, 1: 1}
_DTYPE = {torch.float32: 0, torch.bfloat16: 1}

MODE_FULL, MODE_PARTIAL, MODE_REFRESH = 0, 1, 2

EXPORTS = ["specpv_workspace_bytes", "specpv_block_summarize", "specpv_select_blocks",
           "specpv_partial_verify_attn", "specpv_partial_verify_attn_static", "specpv_full_verify_refresh", "specpv_gather_blocks", "specpv_select_mode",
           "specpv_extend_parents", "specpv_commit_accepted", "specpv_commit_accepted_layers", "specpv_strerror",
           "specpv_last_hip_error", "specpv_version", "specpv_debug_set_route", "specpv_debug_set_select_route",
           "specpv_debug_set_timeline"]


class SpecPVError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("specpv status %d: %s" % (status, text))
        self.status = status


class _KV(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64), ("stride_t", ctypes.c_int64),
                ("ctx_len", ctypes.c_void_p),
                ("batch", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("block_size", ctypes.c_int32), ("max_blocks", ctypes.c_int32), ("dtype", ctypes.c_int)]


class _Tree(ctypes.Structure):
    _fields_ = [("q", ctypes.c_void_p), ("kd", ctypes.c_void_p), ("vd", ctypes.c_void_p),
                ("parent", ctypes.c_void_p), ("M", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("last_node", ctypes.c_int32), ("n_key_only", ctypes.c_int32)]


class _Lists(ctypes.Structure):
    _fields_ = [("sel_idx", ctypes.c_void_p), ("sel_count", ctypes.c_void_p), ("n_sel", ctypes.c_int32)]


class _Policy(ctypes.Structure):
    _fields_ = [("partial_budget_tokens", ctypes.c_int32), ("pending_margin_tokens", ctypes.c_int32)]


class _Cfg(ctypes.Structure):
    _fields_ = [("n_sink_blocks", ctypes.c_int32), ("n_recent_blocks", ctypes.c_int32),
                ("k_blocks", ctypes.c_int32), ("reduce", ctypes.c_int), ("score", ctypes.c_int),
                ("n_extra_slots", ctypes.c_int32)]


_lib = None


def lib_path():
    return _LIB_PATH


def load():
    """dlopen libspecpv.so.  Raises if it has not been built: there is no fallback."""
    global _lib, _LIB_PATH
    if _lib is not None:
        return _lib
    # SPECPV_LIB names another build of the same library (the instrumented one that timeline.py measures with)
    _LIB_PATH = os.environ.get("SPECPV_LIB") or _LIB_PATH
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError("libspecpv.so is not built (%s missing): run "
                           "`python -m paper_2512_02337_amd.build` first" % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    P = ctypes.POINTER
    lib.specpv_workspace_bytes.restype = sz
    lib.specpv_workspace_bytes.argtypes = [P(_KV), P(_Tree), P(_Cfg)]
    lib.specpv_block_summarize.restype = ctypes.c_int
    lib.specpv_block_summarize.argtypes = [P(_KV), i32, i32, vp, vp, vp]
    lib.specpv_select_blocks.restype = ctypes.c_int
    lib.specpv_select_blocks.argtypes = [P(_KV), P(_Tree), vp, vp, P(_Cfg), vp, vp, vp, vp, sz, vp]
    lib.specpv_partial_verify_attn.restype = ctypes.c_int
    lib.specpv_partial_verify_attn.argtypes = [P(_KV), P(_Tree), vp, vp, i32, vp, vp, vp, sz, vp]
    lib.specpv_partial_verify_attn_static.restype = ctypes.c_int
    lib.specpv_partial_verify_attn_static.argtypes = [P(_KV), P(_Tree), vp, vp, i32, vp, vp, vp]
    lib.specpv_full_verify_refresh.restype = ctypes.c_int
    lib.specpv_full_verify_refresh.argtypes = [P(_KV), P(_Tree), vp, vp, i32, P(_Cfg), vp, vp, vp, vp, vp, vp, sz, vp]
    lib.specpv_gather_blocks.restype = ctypes.c_int
    lib.specpv_gather_blocks.argtypes = [P(_KV), vp, vp, i32, vp, vp, vp, vp]
    lib.specpv_select_mode.restype = ctypes.c_int
    lib.specpv_select_mode.argtypes = [P(_Policy), ctypes.c_int64, i32, i32]
    lib.specpv_extend_parents.restype = ctypes.c_int
    lib.specpv_extend_parents.argtypes = [P(i32), i32, i32, P(i32)]
    lib.specpv_commit_accepted.restype = ctypes.c_int
    lib.specpv_commit_accepted.argtypes = [P(_KV), vp, vp, i32, i32, vp, vp, vp, i32, ctypes.c_int, vp, vp,
                                           P(_Lists), vp, vp, sz, vp]
    lib.specpv_commit_accepted_layers.restype = ctypes.c_int
    lib.specpv_commit_accepted_layers.argtypes = [P(P(_KV)), P(vp), P(vp), i32, i32, i32, vp, vp, vp, i32, ctypes.c_int,
                                                  P(vp), P(vp), P(_Lists), vp, vp, sz, vp]
    lib.specpv_debug_set_route.restype = ctypes.c_int
    lib.specpv_debug_set_route.argtypes = [ctypes.c_int]
    lib.specpv_debug_set_select_route.restype = ctypes.c_int
    lib.specpv_debug_set_select_route.argtypes = [ctypes.c_int]
    lib.specpv_strerror.restype = ctypes.c_char_p
    lib.specpv_strerror.argtypes = [ctypes.c_int]
    lib.specpv_last_hip_error.restype = ctypes.c_char_p
    lib.specpv_version.restype = ctypes.c_int
    _lib = lib
    return lib


def _check(rc):
    if rc != 0:
        lib = load()
        text = lib.specpv_strerror(rc).decode()
        if rc == -4:
            text += " [" + lib.specpv_last_hip_error().decode() + "]"
        raise SpecPVError(rc, text)


def _ptr(t, dtype=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("%s must live on the GPU" % name)
    if dtype is not None and t.dtype != dtype:
        raise ValueError("%s must be %s, is %s" % (name, dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


class KV:
    """One layer's committed KV cache (descriptor `specpv_kv`).
    k, v: [batch, Hkv, T, D] (head-major, layout="bhtd") or [batch, T, Hkv, D]
    (token-major, layout="bthd"); T >= max_blocks * block_size is not required,
    only rows t < ctx_len[b] are read.  ctx_len: int32 [batch] on the GPU."""

    def __init__(self, k, v, ctx_len, block_size, max_blocks=None, layout="bhtd"):
        if k.dtype not in _DTYPE or v.dtype != k.dtype or k.shape != v.shape or k.dim() != 4:
            raise ValueError("k, v: same 4-d shape, float32 or bfloat16")
        if k.stride() != v.stride() or k.stride(3) != 1:
            raise ValueError("k and v must share strides; the head dim must be contiguous")
        if layout == "bhtd":
            batch, hkv, T, D = k.shape
            sb, sh, st = k.stride(0), k.stride(1), k.stride(2)
        elif layout == "bthd":
            batch, T, hkv, D = k.shape
            sb, st, sh = k.stride(0), k.stride(1), k.stride(2)
        else:
            raise ValueError(layout)
        self.k, self.v, self.ctx_len = k, v, ctx_len
        self.batch, self.Hkv, self.T, self.D, self.B = batch, hkv, T, D, int(block_size)
        self.max_blocks = int(max_blocks) if max_blocks is not None else (T + self.B - 1) // self.B
        if self.max_blocks * self.B > T + self.B - 1:
            raise ValueError("max_blocks exceeds the allocated rows")
        if ctx_len.dtype != torch.int32 or ctx_len.numel() != batch:
            raise ValueError("ctx_len: int32 [batch]")
        self.dtype = k.dtype
        self.c = _KV(k.data_ptr(), v.data_ptr(), sb, sh, st, _ptr(ctx_len, torch.int32, "ctx_len").value,
                     batch, hkv, D, self.B, self.max_blocks, _DTYPE[k.dtype])

    def summary_shape(self):
        return (self.batch, self.Hkv, self.max_blocks, self.D)


class Tree:
    """The draft tree of one verify step (descriptor `specpv_tree`).
    kd, vd [batch, M, Hkv, D]; parent int32 [batch, M]; q [batch, Mq, Hq, D] with Mq <= M: the
    first M - Mq nodes are keys only (the partially verified tokens on a partial step)."""

    def __init__(self, q, kd=None, vd=None, parent=None, last_node=None):
        if q.dim() != 4:
            raise ValueError("q: [batch, Mq, Hq, D]")
        self.q, self.kd, self.vd, self.parent = q, kd, vd, parent
        self.batch, self.Mq, self.Hq, self.D = q.shape
        self.M = self.Mq
        for t in (kd, vd):
            if t is not None:
                self.M = t.shape[1]
        if parent is not None:
            self.M = parent.shape[1]
        if self.M < self.Mq:
            raise ValueError("fewer tree nodes than query rows")
        self.n_key_only = self.M - self.Mq
        for name, t in (("kd", kd), ("vd", vd)):
            if t is not None and (t.dtype != q.dtype or tuple(t.shape[:2]) != (self.batch, self.M) or t.shape[3] != q.shape[3]):
                raise ValueError("%s: [batch, M, Hkv, D] in q's dtype" % name)
        if parent is not None and (parent.dtype != torch.int32 or tuple(parent.shape) != (self.batch, self.M)):
            raise ValueError("parent: int32 [batch, M]")
        self.c = _Tree(_ptr(q, None, "q").value,
                       None if kd is None else _ptr(kd, q.dtype, "kd").value,
                       None if vd is None else _ptr(vd, q.dtype, "vd").value,
                       None if parent is None else _ptr(parent, torch.int32, "parent").value,
                       self.M, self.Hq, self.n_key_only if last_node is None else int(last_node), self.n_key_only)


class SelectCfg:
    def __init__(self, n_sink_blocks, n_recent_blocks, k_blocks, reduce="mean", score="eq2", n_extra_slots=0):
        self.ns, self.nr, self.k = int(n_sink_blocks), int(n_recent_blocks), int(k_blocks)
        self.n_extra = int(n_extra_slots)
        self.n_sel = self.ns + self.k + self.nr + self.n_extra     # entries per list row
        self.c = _Cfg(self.ns, self.nr, self.k, _REDUCE[reduce], _SCORE[score], self.n_extra)


def _match(kv, tree):
    if tree.q.dtype != kv.dtype or tree.D != kv.D or tree.batch != kv.batch:
        raise ValueError("tree and kv disagree in dtype, head dim or batch")
    if tree.kd is not None and tree.kd.shape[2] != kv.Hkv:
        raise ValueError("kd / vd must have Hkv heads")


def specpv_workspace_bytes(kv, tree=None, cfg=None):
    return int(load().specpv_workspace_bytes(ctypes.byref(kv.c), None if tree is None else ctypes.byref(tree.c),
                                             None if cfg is None else ctypes.byref(cfg.c)))


def specpv_block_summarize(kv, blk_begin, blk_end, kmax, kmin):
    for name, t in (("kmax", kmax), ("kmin", kmin)):
        if tuple(t.shape) != kv.summary_shape():
            raise ValueError("%s: [batch, Hkv, max_blocks, D]" % name)
    _check(load().specpv_block_summarize(ctypes.byref(kv.c), int(blk_begin), int(blk_end),
                                         _ptr(kmax, kv.dtype, "kmax"), _ptr(kmin, kv.dtype, "kmin"), _stream()))


def _ws(workspace):
    if workspace is None:
        return None, 0
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous GPU tensor")
    return ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()


def _check_sel(kv, sel_idx, sel_count, n_sel):
    if tuple(sel_idx.shape) != (kv.batch, kv.Hkv, n_sel) or tuple(sel_count.shape) != (kv.batch, kv.Hkv):
        raise ValueError("sel_idx [batch, Hkv, n_sel], sel_count [batch, Hkv]")


def specpv_select_blocks(kv, tree, kmax, kmin, cfg, sel_idx, sel_count, scores=None, workspace=None):
    _match(kv, tree)
    _check_sel(kv, sel_idx, sel_count, cfg.n_sel)
    if scores is not None and tuple(scores.shape) != (kv.batch, kv.Hkv, kv.max_blocks):
        raise ValueError("scores: [batch, Hkv, max_blocks] float32")
    for name, t in (("kmax", kmax), ("kmin", kmin)):
        if tuple(t.shape) != kv.summary_shape():
            raise ValueError("%s: [batch, Hkv, max_blocks, D]" % name)
    wp, wb = _ws(workspace)
    _check(load().specpv_select_blocks(ctypes.byref(kv.c), ctypes.byref(tree.c), _ptr(kmax, kv.dtype, "kmax"),
                                       _ptr(kmin, kv.dtype, "kmin"), ctypes.byref(cfg.c),
                                       _ptr(sel_idx, torch.int32, "sel_idx"), _ptr(sel_count, torch.int32, "sel_count"),
                                       _ptr(scores, torch.float32, "scores"), wp, wb, _stream()))


def specpv_partial_verify_attn(kv, tree, sel_idx, sel_count, out, lse=None, workspace=None):
    _match(kv, tree)
    n_sel = 0
    if sel_idx is not None:
        n_sel = sel_idx.shape[-1]
        _check_sel(kv, sel_idx, sel_count, n_sel)
    if out.shape != tree.q.shape:
        raise ValueError("out: same shape as q")
    if lse is not None and tuple(lse.shape) != (tree.batch, tree.Mq, tree.Hq):
        raise ValueError("lse: [batch, Mq, Hq] float32")
    wp, wb = _ws(workspace)
    _check(load().specpv_partial_verify_attn(ctypes.byref(kv.c), ctypes.byref(tree.c),
                                             _ptr(sel_idx, torch.int32, "sel_idx"),
                                             _ptr(sel_count, torch.int32, "sel_count"), n_sel,
                                             _ptr(out, kv.dtype, "out"), _ptr(lse, torch.float32, "lse"),
                                             wp, wb, _stream()))


def specpv_partial_verify_attn_static(kv, tree, sel_idx, sel_count, out, lse=None):
    """specpv_partial_verify_attn without a workspace: the partial results live in the library's own
    static device array (at most STATIC_SCRATCH_BYTES; larger shapes raise SpecPVError -3)."""
    _match(kv, tree)
    n_sel = 0
    if sel_idx is not None:
        n_sel = sel_idx.shape[-1]
        _check_sel(kv, sel_idx, sel_count, n_sel)
    if out.shape != tree.q.shape:
        raise ValueError("out: same shape as q")
    if lse is not None and tuple(lse.shape) != (tree.batch, tree.Mq, tree.Hq):
        raise ValueError("lse: [batch, Mq, Hq] float32")
    rc = load().specpv_partial_verify_attn_static(ctypes.byref(kv.c), ctypes.byref(tree.c),
                                                  _ptr(sel_idx, torch.int32, "sel_idx"),
                                                  _ptr(sel_count, torch.int32, "sel_count"), n_sel,
                                                  _ptr(out, kv.dtype, "out"), _ptr(lse, torch.float32, "lse"), _stream())
    if rc == -3:
        raise SpecPVError(rc, load().specpv_strerror(rc).decode() + " [" + load().specpv_last_hip_error().decode() + "]")
    _check(rc)


STATIC_SCRATCH_BYTES = 16 << 20


def specpv_full_verify_refresh(kv, tree, kmax, kmin, stale_blk_begin, cfg, out, lse, sel_idx, sel_count,
                               scores=None, workspace=None):
    _match(kv, tree)
    _check_sel(kv, sel_idx, sel_count, cfg.n_sel)
    if out.shape != tree.q.shape:
        raise ValueError("out: same shape as q")
    for name, t in (("kmax", kmax), ("kmin", kmin)):
        if tuple(t.shape) != kv.summary_shape():
            raise ValueError("%s: [batch, Hkv, max_blocks, D]" % name)
    if lse is not None and tuple(lse.shape) != (tree.batch, tree.Mq, tree.Hq):
        raise ValueError("lse: [batch, Mq, Hq] float32")
    if scores is not None and tuple(scores.shape) != (kv.batch, kv.Hkv, kv.max_blocks):
        raise ValueError("scores: [batch, Hkv, max_blocks] float32")
    wp, wb = _ws(workspace)
    _check(load().specpv_full_verify_refresh(ctypes.byref(kv.c), ctypes.byref(tree.c), _ptr(kmax, kv.dtype, "kmax"),
                                             _ptr(kmin, kv.dtype, "kmin"), int(stale_blk_begin), ctypes.byref(cfg.c),
                                             _ptr(out, kv.dtype, "out"), _ptr(lse, torch.float32, "lse"),
                                             _ptr(sel_idx, torch.int32, "sel_idx"),
                                             _ptr(sel_count, torch.int32, "sel_count"),
                                             _ptr(scores, torch.float32, "scores"), wp, wb, _stream()))


def specpv_gather_blocks(kv, sel_idx, sel_count, out_k, out_v, out_len=None):
    """out_k / out_v [batch, Hkv, n_sel * B, D]; out_len int32 [batch] (optional)."""
    n_sel = sel_idx.shape[-1]
    _check_sel(kv, sel_idx, sel_count, n_sel)
    for name, t in (("out_k", out_k), ("out_v", out_v)):
        if tuple(t.shape) != (kv.batch, kv.Hkv, n_sel * kv.B, kv.D):
            raise ValueError("%s: [batch, Hkv, n_sel * B, D]" % name)
    _check(load().specpv_gather_blocks(ctypes.byref(kv.c), _ptr(sel_idx, torch.int32, "sel_idx"),
                                       _ptr(sel_count, torch.int32, "sel_count"), n_sel, _ptr(out_k, kv.dtype, "out_k"),
                                       _ptr(out_v, kv.dtype, "out_v"), _ptr(out_len, torch.int32, "out_len"), _stream()))


def specpv_select_mode(partial_budget_tokens, pending_margin_tokens, seq_len, partial_ready, n_pending):
    pol = _Policy(int(partial_budget_tokens), int(pending_margin_tokens))
    rc = load().specpv_select_mode(ctypes.byref(pol), int(seq_len), 1 if partial_ready else 0, int(n_pending))
    if rc < 0:
        _check(rc)
    return rc


def specpv_extend_parents(tree_parent, n_pending):
    """tree_parent: sequence of M_tree ints (host).  Returns the n_pending + M_tree parents as a list."""
    m = len(tree_parent)
    src = (ctypes.c_int32 * m)(*[int(x) for x in tree_parent])
    dst = (ctypes.c_int32 * (m + int(n_pending)))()
    _check(load().specpv_extend_parents(src, m, int(n_pending), dst))
    return list(dst)


def _lists(kv, sel_idx, sel_count):
    n_sel = sel_idx.shape[-1]
    _check_sel(kv, sel_idx, sel_count, n_sel)
    return _Lists(_ptr(sel_idx, torch.int32, "sel_idx").value, _ptr(sel_count, torch.int32, "sel_count").value, n_sel)


def _dropped(kv, dropped):
    if dropped is not None and tuple(dropped.shape) != (kv.batch, 2):
        raise ValueError("dropped: int32 [batch, 2]")
    return _ptr(dropped, torch.int32, "dropped")


def specpv_commit_accepted(kv, buf_k, buf_v, pending_cap, M_tree, n_pending, accepted, n_accepted, mode,
                           kmax=None, kmin=None, workspace=None, sel_idx=None, sel_count=None, dropped=None):
    """buf_k / buf_v [batch, pending_cap + M_tree, Hkv, D]; n_pending, n_accepted int32 [batch];
    accepted int32 [batch, max_accept]; optional sel_idx / sel_count (the layer's kept-block lists, extended
    by a commit to the cache) and dropped int32 [batch, 2] -- all on the GPU."""
    for name, t in (("buf_k", buf_k), ("buf_v", buf_v)):
        if tuple(t.shape) != (kv.batch, pending_cap + M_tree, kv.Hkv, kv.D):
            raise ValueError("%s: [batch, pending_cap + M_tree, Hkv, D]" % name)
    if tuple(n_pending.shape) != (kv.batch,) or tuple(n_accepted.shape) != (kv.batch,) or accepted.dim() != 2 \
            or accepted.shape[0] != kv.batch:
        raise ValueError("n_pending, n_accepted: int32 [batch]; accepted: int32 [batch, max_accept]")
    for name, t in (("kmax", kmax), ("kmin", kmin)):
        if t is not None and tuple(t.shape) != kv.summary_shape():
            raise ValueError("%s: [batch, Hkv, max_blocks, D]" % name)
    wp, wb = _ws(workspace)
    ls = None if sel_idx is None else ctypes.byref(_lists(kv, sel_idx, sel_count))
    _check(load().specpv_commit_accepted(ctypes.byref(kv.c), _ptr(buf_k, kv.dtype, "buf_k"), _ptr(buf_v, kv.dtype, "buf_v"),
                                         int(pending_cap), int(M_tree), _ptr(n_pending, torch.int32, "n_pending"),
                                         _ptr(accepted, torch.int32, "accepted"), _ptr(n_accepted, torch.int32, "n_accepted"),
                                         int(accepted.shape[1]), int(mode), _ptr(kmax, kv.dtype, "kmax"),
                                         _ptr(kmin, kv.dtype, "kmin"), ls, _dropped(kv, dropped), wp, wb, _stream()))


def specpv_commit_accepted_layers(kvs, buf_ks, buf_vs, pending_cap, M_tree, n_pending, accepted, n_accepted, mode,
                                  kmaxs=None, kmins=None, workspace=None, sel_idxs=None, sel_counts=None, dropped=None):
    """specpv_commit_accepted for all layers of a model at once: kvs, buf_ks, buf_vs (and kmaxs, kmins,
    sel_idxs, sel_counts) are lists with one entry per layer; the layers share shape, strides, dtype and
    ONE ctx_len tensor."""
    n = len(kvs)
    if n < 1 or len(buf_ks) != n or len(buf_vs) != n:
        raise ValueError("one kv, buf_k and buf_v per layer")
    kv0 = kvs[0]
    for t in list(buf_ks) + list(buf_vs):
        if tuple(t.shape) != (kv0.batch, pending_cap + M_tree, kv0.Hkv, kv0.D):
            raise ValueError("buffers: [batch, pending_cap + M_tree, Hkv, D]")
    if tuple(n_pending.shape) != (kv0.batch,) or tuple(n_accepted.shape) != (kv0.batch,) or accepted.dim() != 2 \
            or accepted.shape[0] != kv0.batch:
        raise ValueError("n_pending, n_accepted: int32 [batch]; accepted: int32 [batch, max_accept]")
    if (kmaxs is None) != (kmins is None) or (kmaxs is not None and (len(kmaxs) != n or len(kmins) != n)):
        raise ValueError("kmaxs, kmins: both or neither, one per layer")
    for t in list(kmaxs or []) + list(kmins or []):
        if tuple(t.shape) != kv0.summary_shape():
            raise ValueError("summaries: [batch, Hkv, max_blocks, D]")
    kv_arr = (ctypes.POINTER(_KV) * n)(*[ctypes.pointer(k.c) for k in kvs])
    vp = ctypes.c_void_p

    def table(ts, name):
        return (vp * n)(*[_ptr(t, kv0.dtype, name) for t in ts])
    bk, bv = table(buf_ks, "buf_k"), table(buf_vs, "buf_v")
    km = table(kmaxs, "kmax") if kmaxs is not None else None
    kn = table(kmins, "kmin") if kmins is not None else None
    wp, wb = _ws(workspace)
    ls = None
    if sel_idxs is not None:
        if len(sel_idxs) != n or len(sel_counts) != n:
            raise ValueError("sel_idxs, sel_counts: one per layer")
        ls = (_Lists * n)(*[_lists(kv0, a, c) for a, c in zip(sel_idxs, sel_counts)])
    _check(load().specpv_commit_accepted_layers(kv_arr, bk, bv, n, int(pending_cap), int(M_tree),
                                                _ptr(n_pending, torch.int32, "n_pending"),
                                                _ptr(accepted, torch.int32, "accepted"),
                                                _ptr(n_accepted, torch.int32, "n_accepted"), int(accepted.shape[1]),
                                                int(mode), km, kn, ls, _dropped(kv0, dropped), wp, wb, _stream()))


def specpv_debug_set_timeline(buf):
    """buf: int64 GPU tensor of 16 entries per workgroup, or None."""
    lib = load()
    lib.specpv_debug_set_timeline.argtypes = [ctypes.c_void_p]
    lib.specpv_debug_set_timeline.restype = ctypes.c_int
    _check(lib.specpv_debug_set_timeline(None if buf is None else ctypes.c_void_p(buf.data_ptr())))


def specpv_debug_set_route(route):
    _check(load().specpv_debug_set_route(int(route)))


def specpv_debug_set_select_route(route):
    _check(load().specpv_debug_set_select_route(int(route)))


def specpv_strerror(status):
    return load().specpv_strerror(int(status)).decode()


def specpv_version():
    return int(load().specpv_version())
