"""Shared helpers of the GPU parity tests: run the library on a workloads case and
the oracle on the same numbers."""
import numpy as np
import torch

import oracle
import workloads

ATOL = {"f32": 1e-5, "bf16": 2e-2}   # max-abs bar on attention outputs, per input dtype
TAU = 1e-3                          # score margin above which the kept list must be bit-identical


def say(*a):
    print(*a, flush=True)


class GpuRun:
    """Device buffers + descriptors of one case."""

    def __init__(self, specpv, case, layout="bhtd", reduce="mean", last_node=0, cfg=None, score="eq2"):
        self.sp, self.case = specpv, case
        dev = case["q"].device
        assert dev.type == "cuda"
        k, v = case["k"], case["v"]
        if layout == "bthd":
            k = k.permute(0, 2, 1, 3).contiguous()
            v = v.permute(0, 2, 1, 3).contiguous()
        self.k, self.v = k, v
        self.kv = specpv.KV(k, v, case["ctx_len"], case["B"], case["max_blocks"], layout=layout)
        self.tree = specpv.Tree(case["q"], case["kd"], case["vd"], case["parent"], last_node=last_node)
        ns, nr, kb = cfg if cfg is not None else (case["ns"], case["nr"], case["k_blocks"])
        self.cfg = specpv.SelectCfg(ns, nr, kb, reduce, score)
        dt = case["q"].dtype
        b, hkv, nbm, D = self.kv.summary_shape()
        self.kmax = torch.zeros((b, hkv, nbm, D), dtype=dt, device=dev)
        self.kmin = torch.zeros((b, hkv, nbm, D), dtype=dt, device=dev)
        self.scores = torch.zeros((b, hkv, nbm), dtype=torch.float32, device=dev)
        self.sel_idx = torch.full((b, hkv, self.cfg.n_sel), -7, dtype=torch.int32, device=dev)
        self.sel_count = torch.full((b, hkv), -7, dtype=torch.int32, device=dev)
        self.out = torch.zeros_like(case["q"])
        self.lse = torch.zeros(case["q"].shape[:3], dtype=torch.float32, device=dev)
        nbytes = specpv.specpv_workspace_bytes(self.kv, self.tree, self.cfg)
        assert nbytes > 0
        self.ws = torch.zeros((nbytes,), dtype=torch.uint8, device=dev)

    def summarize(self, lo=0, hi=-1):
        self.sp.specpv_block_summarize(self.kv, lo, hi, self.kmax, self.kmin)

    def select(self):
        self.sp.specpv_select_blocks(self.kv, self.tree, self.kmax, self.kmin, self.cfg,
                                     self.sel_idx, self.sel_count, self.scores, self.ws)

    def attend(self, sel_idx="own", sel_count=None):
        if isinstance(sel_idx, str):
            sel_idx, sel_count = self.sel_idx, self.sel_count
        self.sp.specpv_partial_verify_attn(self.kv, self.tree, sel_idx, sel_count, self.out, self.lse, self.ws)

    def refresh(self, stale=0):
        self.sp.specpv_full_verify_refresh(self.kv, self.tree, self.kmax, self.kmin, stale, self.cfg, self.out,
                                           self.lse, self.sel_idx, self.sel_count, self.scores, self.ws)


def oracle_select(case, b, reduce="mean", last_node=0, cfg=None, score="eq2"):
    o = workloads.oracle_views(case, b)
    ns, nr, kb = cfg if cfg is not None else (case["ns"], case["nr"], case["k_blocks"])
    kmax, kmin = oracle.block_summarize(o["K"], case["B"])
    sc = oracle.block_scores(o["Q"], kmax, kmin, reduce, last_node, score)
    idx, cnt = oracle.select_blocks(sc, ns, nr, kb)
    return o, kmax, kmin, sc, idx, cnt


def topk_margin(sc, ns, nr, k):
    """Per KV head: gap between the k-th and (k+1)-th candidate score (inf if all kept)."""
    Hkv, nb = sc.shape
    if nb <= ns + nr + k or k == 0:
        return np.full((Hkv,), np.inf)
    cand = np.sort(sc[:, ns:nb - nr].astype(np.float32).astype(np.float64), axis=1)[:, ::-1]
    return cand[:, k - 1] - cand[:, k]


def check_selection(got_idx, got_cnt, ref_idx, ref_cnt, sc, ns, nr, k, tag=""):
    """Bit-exact where the margin allows; otherwise only blocks whose oracle score
    lies within TAU of the threshold may differ.  Returns True if bit-exact."""
    margin = topk_margin(sc, ns, nr, k)
    exact = True
    for g in range(sc.shape[0]):
        a = got_idx[g, :got_cnt[g]].tolist()
        r = ref_idx[g, :ref_cnt[g]].tolist()
        assert got_cnt[g] == ref_cnt[g], (tag, g, got_cnt[g], ref_cnt[g])
        assert a == sorted(a) and len(set(a)) == len(a), (tag, g, "not ascending / unique")
        assert (got_idx[g, got_cnt[g]:] == -1).all(), (tag, g, "padding")
        if a == r:
            continue
        assert margin[g] <= TAU, (tag, g, "lists differ although margin %.3g > tau" % margin[g], a, r)
        exact = False
        cand = np.sort(sc[g, ns:sc.shape[1] - nr].astype(np.float32))[::-1]
        thr = cand[k - 1]
        for i in set(a) ^ set(r):
            assert abs(np.float32(sc[g, i]) - thr) <= TAU, (tag, g, i, "differs beyond the near-tie band")
    return exact


def with_pending(base, n_key, seed):
    """The case with n_key partially verified tokens (a chain, Section 3.3) in front of every sequence's tree."""
    gen = torch.Generator().manual_seed(seed)
    dt = base["q"].dtype
    bsz = base["batch"]
    pk = torch.randn((bsz, n_key, base["Hkv"], base["D"]), generator=gen).to(dt)
    pv = torch.randn((bsz, n_key, base["Hkv"], base["D"]), generator=gen).to(dt)
    case = dict(base)
    case["kd"], case["vd"] = torch.cat([pk, base["kd"]], 1), torch.cat([pv, base["vd"]], 1)
    case["parent"] = torch.from_numpy(np.array([oracle.extend_parents(base["parent"][b].tolist(), n_key) for b in range(bsz)],
                                               dtype=np.int32))
    return case
