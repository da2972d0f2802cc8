"""Scoring + selection (Section 3.2, eq. 2-3 and the top-k) as one launch, whose last workgroup per
(sequence, KV head) selects, against the same as two launches: scores, lists and counts are the same
bit for bit, on fresh inputs in the same buffers call after call (a stale score read across
workgroups would show), with planted ties at the threshold, workgroups past the end of short
sequences, lists of 1024 / 2048 / 4096 blocks, every reducer and both score kinds; the arrival
words are zero after every call.  The two-launch result of the first case is checked against the
oracle, so the comparison is not between two wrong things.  Only the summaries and the queries are
read by these calls: the K / V arrays stay uninitialised."""
import numpy as np
import pytest
import torch

import oracle
from helpers import check_selection, say

pytestmark = pytest.mark.gpu

# tag, ctx, B, M, Hq, Hkv, (ns, nr, k), reduce, score, pool (0: all summaries distinct; n: the candidates'
# summaries are drawn from n distinct rows, so the threshold falls inside a group of equal scores)
CASES = [
    ("one 128K sequence: 2048 blocks, 64 workgroups per KV head", [131072], 64, 60, 32, 8, (1, 8, 55), "mean", "eq2", 0),
    ("the same with ties at the threshold", [131072], 64, 60, 32, 8, (1, 8, 55), "mean", "eq2", 40),
    ("16K: 256 blocks", [16384], 64, 60, 32, 8, (1, 4, 27), "mean", "eq2", 0),
    ("ragged batch of four at G = 5: four tiles per workgroup, workgroups past the end", [32768, 65536, 98304, 131072],
     64, 60, 40, 8, (1, 8, 55), "mean", "eq2", 0),
    ("4096 blocks of 16 tokens, channel-wise bound, max reducer, ties", [65536], 16, 60, 32, 8, (2, 8, 246), "max", "channel_bound", 300),
    ("an empty, a tiny and two longer sequences, last-node reducer", [0, 100, 5000, 40000], 64, 32, 16, 4, (1, 2, 9), "last", "eq2", 0),
    ("fewer blocks than list entries", [1000], 16, 40, 8, 2, (2, 3, 80), "mean", "eq2", 0),
    ("128 nodes: sixteen wavefronts, two row blocks each", [20000], 32, 128, 16, 2, (1, 2, 30), "mean", "eq2", 7),
    ("64 (sequence, KV head) pairs: arrival words eight bytes apart", [3000, 9000, 500, 7000, 9000, 64, 4000, 8000], 64, 40, 32, 8,
     (1, 2, 20), "mean", "eq2", 0),
]


@pytest.fixture
def routes(gpu_lib):
    yield gpu_lib
    gpu_lib.specpv_debug_set_select_route(0)


def _inputs(gen, batch, Hkv, nbm, D, M, Hq, pool, ns):
    kmin = torch.randn((batch, Hkv, nbm, D), generator=gen, device="cuda")
    kmax = kmin + torch.randn((batch, Hkv, nbm, D), generator=gen, device="cuda").abs()
    if pool:
        src = torch.randint(ns, min(ns + pool, nbm), (nbm,), generator=gen, device="cuda")
        src[:ns] = torch.arange(ns, device="cuda")
        kmin, kmax = kmin[:, :, src], kmax[:, :, src]
    q = torch.randn((batch, M, Hq, D), generator=gen, device="cuda")
    return kmax.bfloat16().contiguous(), kmin.bfloat16().contiguous(), q.bfloat16()


@pytest.mark.parametrize("tag,ctx,B,M,Hq,Hkv,sel,reduce,score,pool", CASES)
def test_one_launch_equals_two(routes, tag, ctx, B, M, Hq, Hkv, sel, reduce, score, pool):
    sp = routes
    say("case:", tag)
    D, batch = 128, len(ctx)
    ns, nr, k = sel
    nbm = max(1, (max(ctx) + B - 1) // B)
    gen = torch.Generator(device="cuda").manual_seed(11)
    kv_rows = torch.empty((batch, Hkv, nbm * B, D), dtype=torch.bfloat16, device="cuda")   # never read
    ctx_len = torch.tensor(ctx, dtype=torch.int32, device="cuda")
    kv = sp.KV(kv_rows, kv_rows, ctx_len, B, nbm)
    q = torch.zeros((batch, M, Hq, D), dtype=torch.bfloat16, device="cuda")
    kmax = torch.zeros((batch, Hkv, nbm, D), dtype=torch.bfloat16, device="cuda")
    kmin = torch.zeros_like(kmax)
    tree = sp.Tree(q, last_node=M // 2)
    cfg = sp.SelectCfg(ns, nr, k, reduce, score)
    ws = torch.zeros((sp.specpv_workspace_bytes(kv, tree, cfg),), dtype=torch.uint8, device="cuda")
    res = {}
    for rep in range(3):
        a, b, c = _inputs(gen, batch, Hkv, nbm, D, M, Hq, pool, ns)
        kmax.copy_(a); kmin.copy_(b); q.copy_(c)
        own_scores = rep != 1          # the second round keeps the scores in the workspace
        for route in (2, 1):
            sp.specpv_debug_set_select_route(route)
            idx = torch.full((batch, Hkv, cfg.n_sel), -7, dtype=torch.int32, device="cuda")
            cnt = torch.full((batch, Hkv), -7, dtype=torch.int32, device="cuda")
            scores = torch.full((batch, Hkv, nbm), -7.0, device="cuda") if own_scores else None
            sp.specpv_select_blocks(kv, tree, kmax, kmin, cfg, idx, cnt, scores, ws)
            torch.cuda.synchronize()
            assert int((ws[:65536].view(torch.int64) != 0).sum()) == 0, "arrival words must be zero after a call"
            res[route] = (idx, cnt, scores)
        for name, x, y in zip(("sel_idx", "sel_count", "scores"), res[2], res[1]):
            if x is not None:
                assert torch.equal(x, y), (tag, "round %d: %s differs between the routes" % (rep, name))
        if pool and rep == 0:
            # the ties are there: some kept candidate's score is shared with a candidate that is not kept
            sc, idx, cnt = res[2][2][0, 0].cpu().numpy(), res[2][0][0, 0].cpu().numpy(), int(res[2][1][0, 0])
            nb = (ctx[0] + B - 1) // B
            kept = set(idx[:cnt].tolist())
            out = {float(sc[i]) for i in range(ns, nb - nr) if i not in kept}
            assert any(float(sc[i]) in out for i in kept if ns <= i < nb - nr), "no tie at the threshold: the case tests nothing"
    if tag.startswith("one 128K"):
        # ... and the lists are the oracle's (KV head 0 and the last one, on the last round's inputs)
        idx, cnt, scores = (t.cpu().numpy() for t in res[1])
        for g in (0, Hkv - 1):
            sc = oracle.block_scores(q[0].cpu()[:, g * (Hq // Hkv):(g + 1) * (Hq // Hkv)], kmax[0, g:g + 1].permute(1, 0, 2).cpu(),
                                     kmin[0, g:g + 1].permute(1, 0, 2).cpu(), reduce, M // 2, score)
            ridx, rcnt = oracle.select_blocks(sc, ns, nr, k)
            np.testing.assert_allclose(scores[0, g], sc[0], atol=1e-3, rtol=0)
            exact = check_selection(idx[0, g:g + 1], cnt[0, g:g + 1], ridx, rcnt, sc, ns, nr, k, tag)
            say("   KV head %d against the oracle: %s" % (g, "identical" if exact else "within the near-tie band"))


def test_one_launch_in_a_graph(routes):
    """The one-launch route inside a HIP graph: the arrival words reset themselves (no memset node), so every replay
    -- with new queries and summaries in the captured buffers, and eager work in between -- gives what the two
    eager launches give on the same inputs."""
    sp = routes
    ctx, B, M, Hq, Hkv, D = [40000, 131072, 9000], 64, 60, 32, 8, 128
    batch, nbm = len(ctx), (max(ctx) + B - 1) // B
    gen = torch.Generator(device="cuda").manual_seed(5)
    kv_rows = torch.empty((batch, Hkv, nbm * B, D), dtype=torch.bfloat16, device="cuda")   # never read
    kv = sp.KV(kv_rows, kv_rows, torch.tensor(ctx, dtype=torch.int32, device="cuda"), B, nbm)
    q = torch.zeros((batch, M, Hq, D), dtype=torch.bfloat16, device="cuda")
    kmax = torch.zeros((batch, Hkv, nbm, D), dtype=torch.bfloat16, device="cuda")
    kmin = torch.zeros_like(kmax)
    tree, cfg = sp.Tree(q), sp.SelectCfg(1, 8, 55, "mean")
    ws = torch.zeros((sp.specpv_workspace_bytes(kv, tree, cfg),), dtype=torch.uint8, device="cuda")
    idx = torch.zeros((batch, Hkv, cfg.n_sel), dtype=torch.int32, device="cuda")
    cnt = torch.zeros((batch, Hkv), dtype=torch.int32, device="cuda")
    scores = torch.zeros((batch, Hkv, nbm), device="cuda")

    def call():
        sp.specpv_select_blocks(kv, tree, kmax, kmin, cfg, idx, cnt, scores, ws)

    sp.specpv_debug_set_select_route(1)
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(stream):
        call()
        stream.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            call()
    torch.cuda.synchronize()
    for rep in range(4):
        a, b, c = _inputs(gen, batch, Hkv, nbm, D, M, Hq, 0, 1)
        kmax.copy_(a); kmin.copy_(b); q.copy_(c)              # eager work between the replays
        for t in (idx, cnt, scores):
            t.fill_(-3)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (idx, cnt, scores)]
        assert int((ws[:65536].view(torch.int64) != 0).sum()) == 0, "arrival words must be zero after a replay"
        for t in (idx, cnt, scores):
            t.fill_(-3)
        sp.specpv_debug_set_select_route(2)
        call()
        torch.cuda.synchronize()
        sp.specpv_debug_set_select_route(1)
        for name, x, y in zip(("sel_idx", "sel_count", "scores"), got, (idx, cnt, scores)):
            assert torch.equal(x, y), "replay %d differs from the two eager launches in %s" % (rep, name)


@pytest.mark.parametrize("reduce", ["mean", "max", "last"])
def test_batched_scoring_against_the_oracle(routes, reduce):
    """The scoring kernel that batches take at G = 5 (query rows held in registers over eight tiles of 32 blocks per
    workgroup, Section 3.2 eq. 2-3) against the oracle: scores and kept lists of the shortest and the longest sequence
    of a ragged batch, every reducer (the last wavefront's rows end ragged: 300 rows in ten blocks of 32)."""
    sp = routes
    ctx, B, M, Hq, Hkv, D = [32768, 65536, 98304, 131072], 64, 60, 40, 8, 128
    ns, nr, k = 1, 8, 55
    batch, nbm = len(ctx), (max(ctx) + B - 1) // B
    gen = torch.Generator(device="cuda").manual_seed(29)
    kv_rows = torch.empty((batch, Hkv, nbm * B, D), dtype=torch.bfloat16, device="cuda")   # never read
    kv = sp.KV(kv_rows, kv_rows, torch.tensor(ctx, dtype=torch.int32, device="cuda"), B, nbm)
    kmax, kmin, q = _inputs(gen, batch, Hkv, nbm, D, M, Hq, 0, ns)
    last_node = 37
    tree, cfg = sp.Tree(q, last_node=last_node), sp.SelectCfg(ns, nr, k, reduce)
    ws = torch.zeros((sp.specpv_workspace_bytes(kv, tree, cfg),), dtype=torch.uint8, device="cuda")
    idx = torch.full((batch, Hkv, cfg.n_sel), -7, dtype=torch.int32, device="cuda")
    cnt = torch.full((batch, Hkv), -7, dtype=torch.int32, device="cuda")
    scores = torch.full((batch, Hkv, nbm), -7.0, device="cuda")
    sp.specpv_select_blocks(kv, tree, kmax, kmin, cfg, idx, cnt, scores, ws)
    torch.cuda.synchronize()
    G = Hq // Hkv
    for b, g in ((0, 0), (0, Hkv - 1), (3, 2), (3, Hkv - 1)):
        nb = (ctx[b] + B - 1) // B
        sc = oracle.block_scores(q[b].cpu()[:, g * G:(g + 1) * G], kmax[b, g:g + 1, :nb].permute(1, 0, 2).cpu(),
                                 kmin[b, g:g + 1, :nb].permute(1, 0, 2).cpu(), reduce, last_node, "eq2")
        ridx, rcnt = oracle.select_blocks(sc, ns, nr, k)
        got = scores[b, g, :nb].cpu().numpy()
        np.testing.assert_allclose(got, sc[0], atol=1e-3 * max(1.0, float(np.abs(sc).max()) / 16), rtol=2e-5)
        exact = check_selection(idx[b, g:g + 1].cpu().numpy(), cnt[b, g:g + 1].cpu().numpy(), ridx, rcnt, sc, ns, nr, k,
                                "sequence %d head %d %s" % (b, g, reduce))
        say("   sequence %d KV head %d, %s: %s" % (b, g, reduce, "identical" if exact else "within the near-tie band"))
