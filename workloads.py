"""Seeded synthetic inputs for the SpecPV verification path.

Serves both the CPU oracle's tests and the GPU library's tests / bench, and
holds none of the method's arithmetic: it only draws random tensors, plants
heavy-hitter blocks and builds draft trees.  The inputs stand in for the
long-context workloads of the paper's Section 4 (LLaMA-3.1-8B / Qwen3 attention
shapes, PG-19 / LongBench contexts), of which only the shapes are available:
head counts, head dim, context lengths, block sizes and KV budgets.

Tensors handed out (torch, on the requested device):
  q   [batch, M, Hq, D]          queries of the draft-tree nodes (post-RoPE)
  k,v [batch, Hkv, Lmax, D]      committed context, head-major; sequence b is
                                 valid for t < ctx_len[b], zero beyond
  kd,vd [batch, M, Hkv, D]       keys / values of the draft-tree nodes
  parent [batch, M] int32        parent[0] = -1, parent[i] < i
  ctx_len [batch] int32
Values are N(0,1) drawn in fp32 and then rounded to the storage dtype, so the
oracle (which widens the rounded values to fp64) and the GPU see the same
numbers.
"""
import math

import numpy as np
import torch

# name -> shape of the workload.  sink / recent / k are in blocks.
CONFIGS = {
    # tiny fp32 case the oracle finishes instantly
    "tiny_f32": dict(Hq=4, Hkv=1, D=64, dtype="f32", ctx=[2048], B=16, M=16, tree="uniform",
                     ns=1, nr=1, k=8, planted=[3], beta=2.0, layers=1),
    # LLaMA-3.1-8B attention shape, 16K context, 2048-token budget (64 sink + 256 recent)
    "llama8b_16k": dict(Hq=32, Hkv=8, D=128, dtype="bf16", ctx=[16384], B=64, M=60, tree="bounded",
                        ns=1, nr=4, k=27, rho=[0.05], beta=1.5, layers=1),
    # LLaMA-3.1-8B shape, 128K context, 4096-token budget (64 sink + 512 recent), 32 layers
    "llama8b_128k": dict(Hq=32, Hkv=8, D=128, dtype="bf16", ctx=[131072], B=64, M=60, tree="bounded",
                         ns=1, nr=8, k=55, rho=[0.05], beta=1.5, layers=32),
    # Qwen3-8B shape, 64K context: full verification + refresh of a 4096-token budget
    "qwen8b_refresh_64k": dict(Hq=32, Hkv=8, D=128, dtype="bf16", ctx=[65536], B=64, M=60, tree="bounded",
                               ns=1, nr=8, k=55, rho=[0.05], beta=1.5, layers=1),
    # Qwen3-14B shape, ragged batch of 4
    "qwen14b_batch4": dict(Hq=40, Hkv=8, D=128, dtype="bf16", ctx=[32768, 65536, 98304, 131072], B=64, M=60,
                           tree="bounded", ns=1, nr=8, k=55, rho=[0.02, 0.05, 0.10, 0.20], beta=1.5, layers=1),
    # the paper's own geometry (Appendix D): 16-token blocks, 32 sink, 128 local tokens, 4K budget
    "paper_default_4k": dict(Hq=32, Hkv=8, D=128, dtype="bf16", ctx=[61440], B=16, M=60, tree="bounded",
                             ns=2, nr=8, k=246, rho=[0.05], beta=1.5, layers=1),
}

TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


def case_seed(base, cfg_name, layer, seq):
    idx = list(CONFIGS).index(cfg_name) if cfg_name in CONFIGS else 99
    return int(base) + 1000 * idx + 10 * int(layer) + int(seq)


def make_tree(M, kind, rng, max_depth=7, max_children=4):
    """parent[] of a draft tree built in index order (node 0 = root).
    uniform: parent[i] ~ U[0, i).  bounded: parent uniform among earlier nodes
    that are shallower than max_depth and have fewer than max_children children.
    chain: parent[i] = i-1.  star: parent[i] = 0."""
    parent = np.full((M,), -1, dtype=np.int32)
    depth = np.zeros((M,), dtype=np.int64)
    nchild = np.zeros((M,), dtype=np.int64)
    for i in range(1, M):
        if kind == "uniform":
            p = int(rng.integers(0, i))
        elif kind == "chain":
            p = i - 1
        elif kind == "star":
            p = 0
        elif kind == "bounded":
            ok = [a for a in range(i) if depth[a] < max_depth and nchild[a] < max_children]
            p = int(ok[int(rng.integers(0, len(ok)))])
        else:
            raise ValueError(kind)
        parent[i] = p
        depth[i] = depth[p] + 1
        nchild[p] += 1
    return parent


def _randn(shape, gen, device):
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32)


def make_case(cfg, seed=0, layer=0, device="cpu", M=None, tree=None):
    """Build one layer's inputs for a config (name from CONFIGS or a dict of
    the same keys).  Returns a dict of tensors plus the geometry."""
    name = cfg if isinstance(cfg, str) else cfg.get("name", "custom")
    c = dict(CONFIGS[cfg]) if isinstance(cfg, str) else dict(cfg)
    if M is not None:
        c["M"] = M
    if tree is not None:
        c["tree"] = tree
    Hq, Hkv, D, B, Mn = c["Hq"], c["Hkv"], c["D"], c["B"], c["M"]
    G = Hq // Hkv
    dt = TORCH_DTYPE[c["dtype"]]
    ctx = list(c["ctx"])
    batch = len(ctx)
    Lmax = max(ctx)
    nbmax = (Lmax + B - 1) // B
    Lalloc = nbmax * B
    dev = torch.device(device)
    q = torch.empty((batch, Mn, Hq, D), dtype=dt, device=dev)
    k = torch.zeros((batch, Hkv, Lalloc, D), dtype=dt, device=dev)
    v = torch.zeros((batch, Hkv, Lalloc, D), dtype=dt, device=dev)
    kd = torch.empty((batch, Mn, Hkv, D), dtype=dt, device=dev)
    vd = torch.empty((batch, Mn, Hkv, D), dtype=dt, device=dev)
    parent = np.empty((batch, Mn), dtype=np.int32)
    planted = []
    for b, L in enumerate(ctx):
        s = case_seed(seed, name, layer, b)
        gen = torch.Generator(device=dev)
        gen.manual_seed(s)
        rng = np.random.default_rng(s)
        qb = _randn((Mn, Hq, D), gen, dev).to(dt)
        q[b] = qb
        kd[b] = _randn((Mn, Hkv, D), gen, dev).to(dt)
        vd[b] = _randn((Mn, Hkv, D), gen, dev).to(dt)
        kb = _randn((Hkv, L, D), gen, dev)
        v[b, :, :L] = _randn((Hkv, L, D), gen, dev).to(dt)
        parent[b] = make_tree(Mn, c["tree"], rng)
        # heavy hitters: shift every key of a planted block along the mean query
        # direction of its KV head, so the block's score stands out
        nb = (L + B - 1) // B
        lo, hi = c["ns"], nb - c["nr"]
        ncand = max(hi - lo, 0)
        if "planted" in c:
            npl = min(int(c["planted"][b]), ncand)
        else:
            npl = min(int(round(c["rho"][b] * ncand)), ncand)
        u = qb.float().reshape(Mn, Hkv, G, D).mean(dim=(0, 2))
        u = u / u.norm(dim=-1, keepdim=True).clamp_min(1e-20)
        pl_b = []
        for g in range(Hkv):
            blocks = np.sort(rng.choice(ncand, size=npl, replace=False) + lo) if npl else np.zeros((0,), np.int64)
            pl_b.append(blocks.astype(np.int64))
            for i in blocks:
                t0, t1 = int(i) * B, min((int(i) + 1) * B, L)
                kb[g, t0:t1] += c["beta"] * u[g]
        planted.append(pl_b)
        k[b, :, :L] = kb.to(dt)
        del kb
    return dict(name=name, cfg=c, q=q, k=k, v=v, kd=kd, vd=vd,
                parent=torch.from_numpy(parent).to(dev),
                ctx_len=torch.tensor(ctx, dtype=torch.int32, device=dev),
                planted=planted, batch=batch, Hq=Hq, Hkv=Hkv, G=G, D=D, B=B, M=Mn,
                ns=c["ns"], nr=c["nr"], k_blocks=c["k"], n_sel=c["ns"] + c["k"] + c["nr"],
                max_blocks=nbmax, dtype=c["dtype"])


def oracle_views(case, b):
    """Sequence b of a case in the oracle's layouts (CPU, storage dtype kept):
    Q [M,Hq,D], K,V [L,Hkv,D], Kd,Vd [M,Hkv,D], parent [M]."""
    L = int(case["ctx_len"][b])
    K = case["k"][b, :, :L].permute(1, 0, 2).contiguous().cpu()
    V = case["v"][b, :, :L].permute(1, 0, 2).contiguous().cpu()
    return dict(Q=case["q"][b].cpu(), K=K, V=V, Kd=case["kd"][b].cpu(), Vd=case["vd"][b].cpu(),
                parent=case["parent"][b].cpu().numpy(), L=L)


def to_device(case, device):
    """Copy of a case with every tensor moved to `device` (values unchanged)."""
    out = dict(case)
    for key, val in case.items():
        if torch.is_tensor(val):
            out[key] = val.to(device)
    return out
