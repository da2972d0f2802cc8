"""GPU parity on seeded random shapes: head counts, group sizes, head dims, element types, block
sizes, context lengths (ragged batches, empty and one-token contexts), tree sizes and kinds, budgets
and reducers drawn at random, every call checked against the oracle as in test_gpu_parity.py.
The shapes are all valid inputs; what varies is which kernel, split count and tail handling they
reach."""
import random

import numpy as np
import pytest
import torch

import workloads
from helpers import GpuRun, check_selection, oracle_select, say
from test_gpu_parity import _check_attn, _to_np

pytestmark = pytest.mark.gpu


def _draw(rnd):
    Hkv = rnd.choice([1, 2, 3, 4])
    G = rnd.choice([1, 2, 3, 4, 5, 6, 8])
    dtype = rnd.choice(["bf16", "bf16", "f32"])
    D = rnd.choice([64, 128, 128])
    B = rnd.choice([4, 7, 16, 32, 64])
    batch = rnd.choice([1, 1, 2, 3])
    big = rnd.random() < 0.25 and dtype == "bf16" and D == 128     # long enough for the group kernel
    ctx = []
    for _ in range(batch):
        r = rnd.random()
        if r < 0.08:
            ctx.append(0)
        elif r < 0.16:
            ctx.append(rnd.randint(1, B))
        else:
            ctx.append(rnd.randint(20000, 45000) if big else rnd.randint(B, 3000))
    if max(ctx) == 0:
        ctx[0] = B + 1     # a cache without capacity for a single block is not a valid input
    M = rnd.choice([1, 2, 7, 16, 33, 60, 64, 65, 100, 128]) if not big else rnd.choice([9, 24, 60])
    ns, nr = rnd.randint(0, 3), rnd.randint(0, 4)
    k = rnd.choice([0, 1, 5, 12, 40])
    if ns + nr + k == 0:
        k = 1
    return dict(Hq=Hkv * G, Hkv=Hkv, D=D, dtype=dtype, ctx=ctx, B=B, M=M,
                tree=rnd.choice(["uniform", "bounded", "chain", "star"]), ns=ns, nr=nr, k=k,
                rho=[0.1] * batch, beta=1.5, layers=1, name="random"), rnd.choice(["mean", "max", "last"])


@pytest.mark.parametrize("seed", range(24))
def test_random_shape(gpu_lib, seed):
    rnd = random.Random(1000 + seed)
    cfg, reduce = _draw(rnd)
    last_node = rnd.randrange(cfg["M"])
    layout = rnd.choice(["bhtd", "bthd"])
    say("case", seed, {k: cfg[k] for k in ("Hq", "Hkv", "D", "dtype", "ctx", "B", "M", "tree", "ns", "nr", "k")}, reduce, layout)
    case = workloads.to_device(workloads.make_case(cfg, seed=seed), "cuda")
    run = GpuRun(gpu_lib, case, layout=layout, reduce=reduce, last_node=last_node)
    run.summarize(); run.select(); run.attend()
    torch.cuda.synchronize()
    sel = []
    for b in range(case["batch"]):
        got_idx, got_cnt = run.sel_idx.cpu().numpy()[b], run.sel_count.cpu().numpy()[b]
        if int(case["ctx_len"][b]) > 0:
            o, kmax, kmin, sc, idx, cnt = oracle_select(case, b, reduce, last_node)
            nb = kmax.shape[0]
            assert np.array_equal(_to_np(run.kmax)[b].transpose(1, 0, 2)[:nb], kmax)
            assert np.array_equal(_to_np(run.kmin)[b].transpose(1, 0, 2)[:nb], kmin)
            tol = 2e-5 * max(1.0, float(np.abs(sc).max()))
            np.testing.assert_allclose(run.scores.cpu().numpy()[b][:, :nb], sc, rtol=2e-5, atol=tol)
            check_selection(got_idx, got_cnt, idx, cnt, sc, case["ns"], case["nr"], case["k_blocks"], "seed %d" % seed)
        else:
            assert (got_cnt == 0).all() and (got_idx == -1).all()
        sel.append((got_idx, got_cnt))
    _check_attn(run, case, sel, "seed %d partial" % seed)
    run.out.zero_(); run.lse.zero_()
    run.refresh(stale=0)
    torch.cuda.synchronize()
    _check_attn(run, case, None, "seed %d full" % seed)


@pytest.mark.parametrize("seed", range(16))
def test_random_shape_with_pending_tokens(gpu_lib, seed):
    """The same draws with a chain of partially verified tokens in front of the tree (keys only, Section 3.3):
    the matrix-core kernels attend them as chunks behind the cache tokens, the vector-ALU kernel through the
    combine; empty and one-token contexts, ragged batches, every group size."""
    import oracle
    from helpers import ATOL, with_pending
    rnd = random.Random(5000 + seed)
    cfg, _ = _draw(rnd)
    cfg["M"] = min(cfg["M"], 96)
    n_key = rnd.choice([1, 3, 16, 20, 31, 32, 33, 64][: 8 if cfg["M"] <= 64 else 6])
    layout = rnd.choice(["bhtd", "bthd"])
    say("case", seed, {k: cfg[k] for k in ("Hq", "Hkv", "D", "dtype", "ctx", "B", "M", "tree", "ns", "nr", "k")}, "pending", n_key, layout)
    base = workloads.make_case(cfg, seed=seed)
    case = workloads.to_device(with_pending(base, n_key, 900 + seed), "cuda")
    run = GpuRun(gpu_lib, case, layout=layout, reduce="mean", last_node=n_key)
    assert run.tree.n_key_only == n_key
    run.summarize(); run.select(); run.attend()
    torch.cuda.synchronize()
    for full in (False, True):
        if full:
            run.out.zero_(); run.lse.zero_()
            run.attend(None, None)
            torch.cuda.synchronize()
        out, lse = _to_np(run.out), _to_np(run.lse)
        worst = 0.0
        for b in range(case["batch"]):
            o = workloads.oracle_views(case, b)
            gi, gc = (None, None) if full else (run.sel_idx.cpu().numpy()[b], run.sel_count.cpu().numpy()[b])
            O, LSE, _ = oracle.tree_attention(o["Q"], o["K"], o["V"], o["Kd"], o["Vd"], o["parent"], case["B"], gi, gc,
                                              n_key_only=n_key)
            worst = max(worst, np.abs(out[b] - O).max())
            np.testing.assert_allclose(lse[b], LSE, atol=2e-5 if case["dtype"] == "f32" else 2e-3, rtol=1e-5)
        say("   seed %d %s: max-abs err %.3g" % (seed, "every block" if full else "kept lists", worst))
        assert worst <= ATOL[case["dtype"]]
