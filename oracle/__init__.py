"""CPU fp64 oracle of the SpecPV verification path.  TEST INFRASTRUCTURE ONLY.

Thin ctypes front end of ``specpv_oracle.c`` (plain C loops that follow the
paper's Section 3.2 / 3.3 definitions one by one).  Only ``tests/``, the smoke
check and the bench's ``cpu_baseline`` leg may import this package; the product
package never does, and this package never imports the product.

Every function takes ONE sequence of ONE layer.  Arrays may be numpy arrays or
torch tensors of any float dtype; they are widened to float64 (exactly) before
the C code sees them.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "specpv_oracle.c")
_LIB = os.path.join(_HERE, "libspecpv_oracle.so")

REDUCE_MEAN, REDUCE_MAX, REDUCE_LAST = 0, 1, 2
_REDUCE = {"mean": 0, "max": 1, "last": 2, 0: 0, 1: 1, 2: 2}


_FLAGS = ["-O2"]   # generic x86-64, no -ffast-math: the build the parity tests and the pins use


def build(force=False):
    """Compile specpv_oracle.c with gcc (no -ffast-math, generic x86-64)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    tmp = _LIB + ".tmp%d" % os.getpid()
    subprocess.run(["gcc"] + _FLAGS + ["-fopenmp", "-shared", "-fPIC", "-Wall",
                    "-o", tmp, _SRC, "-lm"], check=True)
    os.replace(tmp, _LIB)
    return _LIB


def use_native_build():
    """Switch this process to a second build of the same source with -O3 -march=native (still no
    -ffast-math: the arithmetic and its order are unchanged), for timing the oracle as a CPU
    baseline on the machine at hand.  The tests keep the generic build."""
    global _LIB, _FLAGS, _lib
    _LIB = os.path.join(_HERE, "libspecpv_oracle_native.so")
    _FLAGS = ["-O3", "-march=native"]
    _lib = None
    build(force=True)   # -march=native must match the machine that runs it


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads():
    return int(_load().oracle_num_threads())


def _f64(x):
    if x is None:
        return None
    if hasattr(x, "detach"):  # torch tensor (bf16 has no numpy dtype: widen first)
        import torch
        x = x.detach().to("cpu").to(torch.float64).numpy()
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64))


def _i32(x):
    if x is None:
        return None
    if hasattr(x, "detach"):
        x = x.detach().to("cpu").numpy()
    return np.ascontiguousarray(np.asarray(x, dtype=np.int32))


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def block_summarize(K, B):
    """eq. 1.  K [L,Hkv,D] -> (kmax, kmin) each [nb,Hkv,D]."""
    K = _f64(K)
    L, Hkv, D = K.shape
    nb = (L + B - 1) // B
    kmax = np.empty((nb, Hkv, D))
    kmin = np.empty((nb, Hkv, D))
    _load().oracle_block_summarize(_p(K), L, Hkv, D, B, _p(kmax), _p(kmin))
    return kmax, kmin


def row_scores(Q, kmax, kmin, score="eq2"):
    """eq. 2 (score="eq2") or the channel-wise bound (score="channel_bound").
    Q [M,Hq,D], summaries [nb,Hkv,D] -> s [Hkv,nb,M*G]."""
    Q, kmax, kmin = _f64(Q), _f64(kmax), _f64(kmin)
    M, Hq, D = Q.shape
    nb, Hkv, _ = kmax.shape
    s = np.empty((Hkv, nb, M * (Hq // Hkv)))
    fn = {"eq2": _load().oracle_row_scores, "channel_bound": _load().oracle_row_scores_channel}[score]
    fn(_p(Q), M, Hq, _p(kmax), _p(kmin), nb, Hkv, D, _p(s))
    return s


def reduce_scores(s, M, G, reduce="mean", last_node=0):
    """eq. 3.  s [Hkv,nb,M*G] -> scores [Hkv,nb]."""
    s = _f64(s)
    Hkv, nb, R = s.shape
    assert R == M * G
    out = np.empty((Hkv, nb))
    _load().oracle_reduce_scores(_p(s), Hkv, nb, M, G, _REDUCE[reduce], int(last_node), _p(out))
    return out


def block_scores(Q, kmax, kmin, reduce="mean", last_node=0, score="eq2"):
    """eq. 2 (or the channel-wise bound) then eq. 3."""
    Q = _f64(Q)
    M, Hq, _ = Q.shape
    Hkv = kmax.shape[1]
    return reduce_scores(row_scores(Q, kmax, kmin, score), M, Hq // Hkv, reduce, last_node)


def select_blocks(scores, ns, nr, k):
    """Sink + top-k + local selection.  scores [Hkv,nb] ->
    (sel_idx [Hkv,ns+k+nr] int32 ascending / -1 padded, sel_count [Hkv])."""
    scores = _f64(scores)
    Hkv, nb = scores.shape
    n_sel = ns + k + nr
    sel_idx = np.empty((Hkv, n_sel), dtype=np.int32)
    sel_count = np.empty((Hkv,), dtype=np.int32)
    _load().oracle_select_blocks(_p(scores), Hkv, nb, ns, nr, k, _p(sel_idx), _p(sel_count))
    return sel_idx, sel_count


def tree_attention(Q, K, V, Kd, Vd, parent, B, sel_idx=None, sel_count=None, n_key_only=0):
    """Tree-masked GQA attention over the kept context blocks plus the draft
    nodes on each node's root path.  sel_idx None = every block (full
    verification).  Returns (O [Mq,Hq,D], lse [Mq,Hq], psum [Mq,Hq]).

    n_key_only: the first n_key_only of the M = len(parent) nodes are keys only (Section 3.2:
    the partially verified tokens wait in the buffer and are attended by the candidates, but a
    partial step does not verify them again): they have rows in Kd / Vd and entries in parent,
    but no query rows; Q holds the Mq = M - n_key_only rows of the other nodes.  The rows of the
    key-only nodes are computed with zero queries and thrown away."""
    Q, K, V, Kd, Vd = _f64(Q), _f64(K), _f64(V), _f64(Kd), _f64(Vd)
    parent = _i32(parent)
    M = parent.shape[0]
    Mq, Hq, D = Q.shape
    assert Mq == M - n_key_only and Kd.shape[0] == M and Vd.shape[0] == M
    if n_key_only:
        Q = np.ascontiguousarray(np.concatenate([np.zeros((n_key_only, Hq, D)), Q]))
    L, Hkv, _ = K.shape
    assert parent[0] == -1 and all(parent[i] < i for i in range(1, M))
    n_sel = 0
    if sel_idx is not None:
        sel_idx, sel_count = _i32(sel_idx), _i32(sel_count)
        n_sel = sel_idx.shape[1]
    O = np.empty((M, Hq, D))
    lse = np.empty((M, Hq))
    psum = np.empty((M, Hq))
    _load().oracle_tree_attention(_p(Q), _p(K), _p(V), _p(Kd), _p(Vd), _p(parent),
                                  M, Hq, Hkv, D, L, B, _p(sel_idx), _p(sel_count),
                                  n_sel, _p(O), _p(lse), _p(psum))
    return O[n_key_only:], lse[n_key_only:], psum[n_key_only:]


def full_verify_refresh(Q, K, V, Kd, Vd, parent, B, ns, nr, k, reduce="mean", last_node=0):
    """Section 3.3: attention over the whole cache, then new summaries, scores
    (with this pass's queries) and a fresh block selection.
    Returns (O, lse, sel_idx, sel_count, scores)."""
    O, lse, _ = tree_attention(Q, K, V, Kd, Vd, parent, B)
    kmax, kmin = block_summarize(K, B)
    scores = block_scores(Q, kmax, kmin, reduce, last_node)
    sel_idx, sel_count = select_blocks(scores, ns, nr, k)
    return O, lse, sel_idx, sel_count, scores


# ---- verification modes and the buffer (Section 3.3; Algorithm 1: SelectMode, PostEvaluate) ----
# Plain Python on one sequence's state; nothing here is shared with the HIP path.
MODE_FULL, MODE_PARTIAL, MODE_REFRESH = 0, 1, 2


def select_mode(seq_len, partial_ready, n_pending, partial_budget_tokens, pending_margin_tokens):
    """Section 3.3: no partial verification while the sequence fits the partial budget; one
    full verification initialises the partial cache once it no longer does; after that
    partial verification, until the partially verified tokens together with one step's
    candidates exceed the buffer (candidates + margin), which triggers a refresh."""
    if seq_len <= partial_budget_tokens:
        return MODE_FULL
    if not partial_ready:
        return MODE_FULL
    if n_pending > pending_margin_tokens:
        return MODE_REFRESH
    return MODE_PARTIAL


def extend_parents(tree_parent, n_pending):
    """Section 3.3: on a refresh the partially verified tokens are prepended to the candidates;
    as a tree they are a chain, and every root of the candidates' tree hangs off its end."""
    out = [i - 1 for i in range(n_pending)]
    for p in tree_parent:
        out.append(n_pending - 1 if p < 0 else int(p) + n_pending)
    return out


def commit_accepted(K, V, L, pend_k, pend_v, cand_k, cand_v, accepted, mode, capacity, pending_cap=None):
    """Sections 3.2 / 3.3, KV side of PostEvaluate for one sequence.
    K, V [capacity, Hkv, D] cache with L committed tokens; pend_k / pend_v: lists of the
    pending tokens' rows [Hkv, D] (oldest first); cand_k / cand_v [M, Hkv, D] this step's
    candidates; accepted: the candidates on the accepted path.  Returns (L, pend_k, pend_v):
    partial verification keeps the accepted candidates as pending tokens; full verification
    and refresh append the pending tokens and then the accepted candidates to the cache.
    Everything else of this step's candidates is dropped.
    Storage is finite: the cache holds `capacity` tokens and the buffer `pending_cap` pending
    tokens (None: unbounded).  Tokens are stored oldest first while there is room; the ones
    that do not fit are lost, and `commit_dropped` says how many that is."""
    rows_k = list(pend_k) + [cand_k[a] for a in accepted]
    rows_v = list(pend_v) + [cand_v[a] for a in accepted]
    if mode == MODE_PARTIAL:
        if pending_cap is not None:
            rows_k, rows_v = rows_k[:pending_cap], rows_v[:pending_cap]
        return L, rows_k, rows_v
    for rk, rv in zip(rows_k, rows_v):
        if L >= capacity:
            break
        K[L] = rk
        V[L] = rv
        L += 1
    return L, [], []


def commit_dropped(L, n_pending, n_accepted, mode, capacity, pending_cap=None):
    """How many of the n_pending + n_accepted tokens `commit_accepted` cannot store."""
    total = n_pending + n_accepted
    if mode == MODE_PARTIAL:
        return 0 if pending_cap is None else max(0, total - pending_cap)
    return max(0, total - max(0, capacity - L))


def extend_lists(sel_idx, sel_count, L_old, L_new, B):
    """Section 3.3 (after a full verification only the invalid tokens are removed, the local
    window is updated): the tokens a full verification / refresh commits stay part of the partial
    cache.  The kept-block lists were built for the length L_old; every block that holds one of
    the tokens L_old .. L_new - 1 joins each head's list (ascending order is kept: these blocks
    lie behind every listed one, except that the first of them may already be listed as the
    ragged last block of the local window).  sel_idx [Hkv, n_sel] (-1 padded), sel_count [Hkv].
    Returns (sel_idx, sel_count, not_listed): new arrays, and per head the number of blocks for
    which the row had no free entry."""
    sel_idx = np.array(sel_idx, dtype=np.int32, copy=True)
    sel_count = np.array(sel_count, dtype=np.int32, copy=True)
    Hkv, n_sel = sel_idx.shape
    not_listed = np.zeros(Hkv, dtype=np.int32)
    if L_new <= L_old:
        return sel_idx, sel_count, not_listed
    first, last = L_old // B, (L_new - 1) // B
    for g in range(Hkv):
        for blk in range(first, last + 1):
            if blk in sel_idx[g, :sel_count[g]].tolist():
                continue
            if sel_count[g] >= n_sel:
                not_listed[g] += 1
                continue
            sel_idx[g, sel_count[g]] = blk
            sel_count[g] += 1
    return sel_idx, sel_count, not_listed


def gather_blocks(K, V, B, sel_idx, sel_count):
    """Section 3.2: the partial cache as a physically contiguous segment.  K, V [L, Hkv, D];
    sel_idx [Hkv, n_sel], sel_count [Hkv].  Returns (Kg, Vg) [n_sel * B, Hkv, D] (rows that no
    kept token fills are zero) and the number of rows filled per head."""
    K, V = _f64(K), _f64(V)
    L, Hkv, D = K.shape
    n_sel = len(sel_idx[0])
    Kg, Vg = np.zeros((n_sel * B, Hkv, D)), np.zeros((n_sel * B, Hkv, D))
    rows = np.zeros(Hkv, dtype=np.int64)
    nb = (L + B - 1) // B
    for g in range(Hkv):
        for slot in range(int(sel_count[g])):
            blk = int(sel_idx[g][slot])
            if blk < 0 or blk >= nb:
                continue
            for r in range(B):
                t = blk * B + r
                if t < L:
                    Kg[slot * B + r, g] = K[t, g]
                    Vg[slot * B + r, g] = V[t, g]
                    rows[g] = max(rows[g], slot * B + r + 1)
    return Kg, Vg, rows
