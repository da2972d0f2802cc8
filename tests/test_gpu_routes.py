"""The routes of specpv_partial_verify_attn (two kernels; one kernel whose last workgroup per row tile
merges the partials; the same with the recompute route forced) all meet the oracle, on shapes with
several splits, empty splits, two row tiles, key-only nodes, ragged batches and lists shorter than
their rows; and the single-kernel route leaves the workspace's arrival words at zero."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from helpers import ATOL, GpuRun, say

pytestmark = pytest.mark.gpu

SMALL = dict(Hq=8, Hkv=2, D=128, dtype="bf16", ctx=[1000], B=16, M=24, tree="bounded",
             ns=2, nr=3, k=9, rho=[0.1], beta=1.5, layers=1, name="small")
CASES = [
    ("llama8b_16k", {}, "headline shape at 16K"),
    (SMALL, {}, "block 16 (chunks cross blocks)"),
    (SMALL, dict(ctx=[100], k=20), "fewer blocks than list entries: splits without tokens"),
    (SMALL, dict(M=100, tree="uniform", B=64, ctx=[3000]), "two row tiles"),
    (SMALL, dict(M=128, tree="chain", ctx=[512]), "root paths of up to 128 nodes"),
    (SMALL, dict(ctx=[640, 1000, 48, 0], rho=[0.1] * 4, B=32), "ragged batch with an empty context"),
    (SMALL, dict(Hq=10, Hkv=2, M=70, B=64, ctx=[2500]), "G = 5, two row tiles"),
]


@pytest.fixture
def routes(gpu_lib):
    yield gpu_lib
    gpu_lib.specpv_debug_set_route(0)


@pytest.mark.parametrize("cfg,over,tag", CASES)
def test_every_route_meets_the_oracle(routes, cfg, over, tag):
    sp = routes
    c = cfg if isinstance(cfg, str) and not over else dict(workloads.CONFIGS[cfg] if isinstance(cfg, str) else cfg, **over)
    case = workloads.to_device(workloads.make_case(c, seed=3), "cuda")
    say("case", tag)
    ref = None
    for route, name in ((1, "two kernels"), (2, "one kernel"), (3, "one kernel, recompute route"), (2, "one kernel again")):
        sp.specpv_debug_set_route(route)
        run = GpuRun(sp, case)
        run.summarize(); run.select()
        run.out.fill_(7.0)
        run.attend()
        torch.cuda.synchronize()
        worst = 0.0
        for b in range(case["batch"]):
            o = workloads.oracle_views(case, b)
            O, LSE, _ = oracle.tree_attention(o["Q"], o["K"], o["V"], o["Kd"], o["Vd"], o["parent"], case["B"],
                                              run.sel_idx.cpu().numpy()[b], run.sel_count.cpu().numpy()[b])
            worst = max(worst, np.abs(run.out[b].float().cpu().numpy() - O).max())
            np.testing.assert_allclose(run.lse[b].cpu().numpy(), LSE, atol=2e-3, rtol=1e-5)
        say("   %-28s max-abs err %.3g" % (name, worst))
        assert worst <= ATOL[case["dtype"]], (tag, name, worst)
        assert int((run.ws[:65536].view(torch.int64) != 0).sum()) == 0, "arrival words must be zero after a call"
        if ref is None:
            ref = run.out.clone()
        else:   # the routes differ only in summation order
            assert (run.out.float() - ref.float()).abs().max().item() <= ATOL[case["dtype"]] * 0.25
        # twice on one workspace: the words reset themselves
        run.out.fill_(-3.0)
        run.attend()
        torch.cuda.synchronize()
        assert (run.out.float() - ref.float()).abs().max().item() <= ATOL[case["dtype"]] * 0.25


def test_single_kernel_route_with_key_only_nodes(routes):
    sp = routes
    base = workloads.make_case("llama8b_16k", seed=3)
    n_key = 13
    gen = torch.Generator().manual_seed(5)
    dt = base["q"].dtype
    pk = torch.randn((1, n_key, base["Hkv"], base["D"]), generator=gen).to(dt)
    pv = torch.randn((1, n_key, base["Hkv"], base["D"]), generator=gen).to(dt)
    case = dict(base)
    case["kd"], case["vd"] = torch.cat([pk, base["kd"]], 1), torch.cat([pv, base["vd"]], 1)
    case["parent"] = torch.from_numpy(np.array([oracle.extend_parents(base["parent"][0].tolist(), n_key)], dtype=np.int32))
    case = workloads.to_device(case, "cuda")
    for route in (2, 3):
        sp.specpv_debug_set_route(route)
        run = GpuRun(sp, case)
        run.summarize(); run.select(); run.attend()
        torch.cuda.synchronize()
        o = workloads.oracle_views(case, 0)
        O, LSE, _ = oracle.tree_attention(o["Q"], o["K"], o["V"], o["Kd"], o["Vd"], o["parent"], case["B"],
                                          run.sel_idx.cpu().numpy()[0], run.sel_count.cpu().numpy()[0], n_key_only=n_key)
        err = np.abs(run.out[0].float().cpu().numpy() - O).max()
        say("   route %d, %d key-only nodes: max-abs err %.3g" % (route, n_key, err))
        assert err <= ATOL["bf16"]
