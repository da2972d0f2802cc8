"""The library's calls inside HIP graphs: the bench times graph replays, so a replay has to
give what the eager calls give, on every replay and with new inputs in the same buffers.
Each graph is replayed several times with eager work (new queries, a new draft tree, new
accepted paths written into the captured buffers) and synchronisations in between, and every
replay is compared bit for bit with the eager calls on the same inputs; the eager result of
the first round is checked against the oracle, so the comparison is not between two wrong
things."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from helpers import ATOL, GpuRun, say, with_pending

pytestmark = pytest.mark.gpu


def _capture(fn):
    """fn captured on a side stream (after one eager warm-up call there); returns the graph."""
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(stream):
        fn()
        stream.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            fn()
    torch.cuda.synchronize()
    return g


def _new_queries(case, seed):
    gen = torch.Generator(device="cuda").manual_seed(seed)
    for name in ("q", "kd", "vd"):
        t = case[name]
        t.copy_(torch.randn(t.shape, generator=gen, device="cuda", dtype=torch.float32).to(t.dtype))
    M = case["M"]
    rng = np.random.default_rng(seed)
    par = np.stack([workloads.make_tree(M, "bounded", rng) for _ in range(case["batch"])])
    case["parent"].copy_(torch.from_numpy(par).to("cuda"))


@pytest.mark.parametrize("name", ["llama8b_16k", "qwen14b_small"])
def test_graph_replays_match_eager(gpu_lib, name):
    if name == "qwen14b_small":   # ragged batch at G = 5 (the ten-wavefront workgroups of the group kernel)
        cfg = dict(workloads.CONFIGS["qwen14b_batch4"])
        cfg.update(ctx=[9000, 33000, 70, 20000], name=name)
    else:
        cfg = name
    case = workloads.to_device(workloads.make_case(cfg, seed=5), "cuda")
    run = GpuRun(gpu_lib, case)
    run.summarize()
    torch.cuda.synchronize()

    def partial_step():
        run.select()
        run.attend()

    def refresh_step():
        run.refresh(stale=-1)

    outs = ("out", "lse", "sel_idx", "sel_count", "scores")
    for tag, step in (("select + partial attention", partial_step), ("full verification + refresh", refresh_step)):
        say("graph:", name, tag)
        g = _capture(step)
        for rep in range(4):
            _new_queries(case, 100 + rep)           # eager work between the replays
            for o in outs:
                getattr(run, o).fill_(-3)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            got = {o: getattr(run, o).clone() for o in outs}
            for o in outs:
                getattr(run, o).fill_(-3)    # same filler: entries that no call writes (blocks past a sequence) compare equal
            step()                                  # the same calls, eagerly, on the same inputs
            torch.cuda.synchronize()
            for o in outs:
                assert torch.equal(got[o], getattr(run, o)), "%s: replay %d differs from the eager calls in %s" % (tag, rep, o)
            if rep == 0:
                # ... and the eager calls are right (sequence 0, against the oracle, on the list the GPU chose)
                c = case
                L = int(c["ctx_len"][0])
                K = c["k"][0, :, :L].permute(1, 0, 2)
                V = c["v"][0, :, :L].permute(1, 0, 2)
                sel = None if step is refresh_step else (run.sel_idx[0].cpu().numpy(), run.sel_count[0].cpu().numpy())
                O, lse, _ = oracle.tree_attention(c["q"][0], K, V, c["kd"][0], c["vd"][0], c["parent"][0], c["B"],
                                                  *(sel if sel else (None, None)))
                err = np.abs(run.out[0].float().cpu().numpy().astype(np.float64) - O).max()
                say("  eager vs oracle: max-abs err %.3g" % err)
                assert err <= ATOL[c["dtype"]]


def test_graph_replays_with_pending_tokens(gpu_lib):
    """A partial step with partially verified tokens in front of the tree (the bench's 16-pending leg): the
    attention kernel takes them as an extra chunk read from the draft K / V arrays."""
    n_key = 16
    base = workloads.make_case("llama8b_16k", seed=5)
    case = workloads.to_device(with_pending(base, n_key, 77), "cuda")
    run = GpuRun(gpu_lib, case)
    run.summarize(); run.select()
    torch.cuda.synchronize()
    g = _capture(run.attend)
    for rep in range(4):
        gen = torch.Generator(device="cuda").manual_seed(300 + rep)
        for name in ("q", "kd", "vd"):   # new queries, new draft and pending K / V rows, same chain + tree
            t = case[name]
            t.copy_(torch.randn(t.shape, generator=gen, device="cuda", dtype=torch.float32).to(t.dtype))
        run.out.fill_(-3); run.lse.fill_(-3)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = run.out.clone(), run.lse.clone()
        run.out.fill_(-3); run.lse.fill_(-3)
        run.attend()
        torch.cuda.synchronize()
        assert torch.equal(got[0], run.out) and torch.equal(got[1], run.lse), "replay %d differs from the eager call" % rep
        if rep == 0:
            o = workloads.oracle_views(case, 0)
            O, lse, _ = oracle.tree_attention(o["Q"], o["K"], o["V"], o["Kd"], o["Vd"], o["parent"], case["B"],
                                              run.sel_idx[0].cpu().numpy(), run.sel_count[0].cpu().numpy(), n_key_only=n_key)
            err = np.abs(run.out[0].float().cpu().numpy().astype(np.float64) - O).max()
            say("  pending tokens, eager vs oracle: max-abs err %.3g" % err)
            assert err <= ATOL[case["dtype"]]


def test_commit_graph_replays_match_eager(gpu_lib):
    """The buffer commit of a partial step in a graph: the counters live on the device and move
    with every replay; a twin state driven by eager calls has to stay identical."""
    sp = gpu_lib
    dev = torch.device("cuda")
    batch, Hkv, D, B, M, P, n_layers = 2, 2, 128, 16, 12, 40, 3
    gen = torch.Generator(device="cuda").manual_seed(7)

    def state():
        st = {"ctx_len": torch.tensor([100, 37], dtype=torch.int32, device=dev),
              "n_pending": torch.zeros((batch,), dtype=torch.int32, device=dev), "kv": [], "bk": [], "bv": []}
        for _ in range(n_layers):
            k = torch.zeros((batch, Hkv, 8 * B, D), dtype=torch.bfloat16, device=dev)
            st["kv"].append(sp.KV(k, torch.zeros_like(k), st["ctx_len"], B, 8))
            st["bk"].append(torch.zeros((batch, P + M, Hkv, D), dtype=torch.bfloat16, device=dev))
            st["bv"].append(torch.zeros_like(st["bk"][-1]))
        return st
    a, b = state(), state()
    accepted = torch.zeros((batch, 4), dtype=torch.int32, device=dev)
    n_accepted = torch.zeros((batch,), dtype=torch.int32, device=dev)
    ws = torch.zeros((1 << 17,), dtype=torch.uint8, device=dev)

    def commit(st):
        sp.specpv_commit_accepted_layers(st["kv"], st["bk"], st["bv"], P, M, st["n_pending"], accepted, n_accepted,
                                         sp.MODE_PARTIAL, None, None, ws)
    snap = {k: [t.clone() for t in a[k]] for k in ("bk", "bv")}
    g = _capture(lambda: commit(a))               # warm-up + capture ran on zero counters: restore the state
    for k in ("bk", "bv"):
        for t, s in zip(a[k], snap[k]):
            t.copy_(s)
    a["n_pending"].zero_()
    for rep in range(5):
        # this step's candidates in the tree part of the buffers, and its accepted path
        for st_bk, st_bv, o_bk, o_bv in zip(a["bk"], a["bv"], b["bk"], b["bv"]):
            new_k = torch.randn((batch, M, Hkv, D), generator=gen, device=dev).to(torch.bfloat16)
            new_v = torch.randn((batch, M, Hkv, D), generator=gen, device=dev).to(torch.bfloat16)
            for bk_, bv_ in ((st_bk, st_bv), (o_bk, o_bv)):
                bk_[:, P:].copy_(new_k)
                bv_[:, P:].copy_(new_v)
        accepted.copy_(torch.tensor([[0, 1 + rep, 7, 9], [0, 2, 3 + rep, 11]], dtype=torch.int32))
        n_accepted.copy_(torch.tensor([1 + rep % 4, 4 - rep % 3], dtype=torch.int32))
        torch.cuda.synchronize()
        g.replay()
        commit(b)
        torch.cuda.synchronize()
        assert torch.equal(a["n_pending"], b["n_pending"]), "replay %d: pending counters" % rep
        for x, y in zip(a["bk"] + a["bv"], b["bk"] + b["bv"]):
            assert torch.equal(x, y), "replay %d: buffer rows" % rep
    assert int(a["n_pending"][0]) == sum(1 + r % 4 for r in range(5))
