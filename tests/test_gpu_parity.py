"""GPU parity: every call of the C ABI against the fp64 oracle, element by element,
on the same seeded inputs.  Bars: summaries and kept-block lists bit-exact (lists
under the near-tie margin rule), attention outputs max-abs <= 1e-5 (fp32 inputs)
or 2e-2 (bf16 inputs)."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from helpers import ATOL, GpuRun, check_selection, oracle_select, say, topk_margin, with_pending

pytestmark = pytest.mark.gpu


def _to_np(t):
    return t.detach().float().cpu().numpy().astype(np.float64) if t.dtype != torch.int32 else t.cpu().numpy()


def _oracle_attn(case, b, sel_idx=None, sel_count=None):
    o = workloads.oracle_views(case, b)
    return oracle.tree_attention(o["Q"], o["K"], o["V"], o["Kd"], o["Vd"], o["parent"], case["B"], sel_idx, sel_count)


def _check_attn(run, case, sel=None, tag="", lse_tol=None):
    """sel: per-sequence list of (idx, cnt) numpy arrays, or None for all blocks."""
    atol = ATOL[case["dtype"]]
    out, lse = _to_np(run.out), _to_np(run.lse)
    worst = 0.0
    for b in range(case["batch"]):
        O, L, ps = _oracle_attn(case, b, *(sel[b] if sel is not None else (None, None)))
        np.testing.assert_allclose(ps, 1.0, atol=1e-12)
        err = np.abs(out[b] - O).max()
        worst = max(worst, err)
        assert err <= atol, (tag, b, "max-abs %.3g > %.3g" % (err, atol))
        np.testing.assert_allclose(lse[b], L, atol=lse_tol or (2e-5 if case["dtype"] == "f32" else 2e-3), rtol=1e-5)
    say("   %s attention max-abs err %.3g (bar %.1g)" % (tag, worst, atol))


@pytest.mark.parametrize("name,seed", [("tiny_f32", 2), ("llama8b_16k", 3)])
def test_whole_path_matches_oracle(gpu_lib, name, seed):
    """summarize -> select -> partial attention, then full verify + refresh."""
    say("case", name, "seed", seed)
    case = workloads.to_device(workloads.make_case(name, seed=seed), "cuda")   # CPU stream: seeds searched offline
    run = GpuRun(gpu_lib, case)
    o, kmax, kmin, sc, idx, cnt = oracle_select(case, 0)
    # eq. 1: bit-exact
    run.summarize()
    torch.cuda.synchronize()
    assert np.array_equal(_to_np(run.kmax)[0].transpose(1, 0, 2), kmax)
    assert np.array_equal(_to_np(run.kmin)[0].transpose(1, 0, 2), kmin)
    # eq. 2-3 + selection
    run.select()
    torch.cuda.synchronize()
    got_sc = run.scores.cpu().numpy()[0]
    np.testing.assert_allclose(got_sc, sc, rtol=2e-5, atol=2e-5)
    margin = topk_margin(sc, case["ns"], case["nr"], case["k_blocks"])
    say("   top-k margins", np.array2string(margin, precision=4))
    assert (margin > 1e-3).all(), "pick a seed whose k-th / (k+1)-th scores are separated"
    assert check_selection(run.sel_idx.cpu().numpy()[0], run.sel_count.cpu().numpy()[0], idx, cnt, sc,
                           case["ns"], case["nr"], case["k_blocks"], name)
    # partial verification attention on the GPU's own list
    run.attend()
    torch.cuda.synchronize()
    _check_attn(run, case, [(idx, cnt)], name + " partial")
    # full verification + refresh, summaries recomputed from block 0
    run.kmax.zero_(); run.kmin.zero_(); run.sel_idx.fill_(-9); run.out.zero_()
    run.refresh(stale=0)
    torch.cuda.synchronize()
    _check_attn(run, case, None, name + " full")
    assert np.array_equal(_to_np(run.kmax)[0].transpose(1, 0, 2), kmax)
    assert check_selection(run.sel_idx.cpu().numpy()[0], run.sel_count.cpu().numpy()[0], idx, cnt, sc,
                           case["ns"], case["nr"], case["k_blocks"], name + " refresh")


SMALL = dict(Hq=8, Hkv=2, D=128, dtype="bf16", ctx=[1000], B=16, M=24, tree="bounded",
             ns=2, nr=3, k=9, rho=[0.1], beta=1.5, layers=1, name="small")


@pytest.mark.parametrize("over,tag", [
    (dict(), "bf16 ragged tail L=1000 B=16"),
    (dict(dtype="f32", D=64), "f32 D=64"),
    (dict(dtype="f32", D=128, B=64, ctx=[1500]), "f32 D=128 B=64"),
    (dict(D=64, ctx=[777], B=32), "bf16 D=64 B=32"),
    (dict(M=1, tree="chain"), "single token decode"),
    (dict(M=128, tree="chain", ctx=[512]), "chain of 128 (refresh-style pending prefix)"),
    (dict(M=100, tree="uniform", Hq=10, Hkv=2), "M=100 G=5"),
    (dict(ctx=[100], k=20), "context shorter than the budget: every block kept"),
    (dict(ctx=[640, 1000, 48, 333], rho=[0.1] * 4), "ragged batch of 4"),
    (dict(ctx=[0, 500], rho=[0.1] * 2), "batch with an empty context (only the draft tokens to attend to)"),
    (dict(Hq=16, Hkv=1), "G=16"),
    (dict(B=7, ctx=[500], ns=3, nr=5, k=11), "odd block size 7"),
])
def test_shapes_and_edges(gpu_lib, over, tag):
    say("case", tag)
    cfg = dict(SMALL); cfg.update(over)
    case = workloads.to_device(workloads.make_case(cfg, seed=11), "cuda")
    for layout in ("bhtd", "bthd"):
        run = GpuRun(gpu_lib, case, layout=layout)
        run.summarize(); run.select(); run.attend()
        torch.cuda.synchronize()
        sel = []
        for b in range(case["batch"]):
            o, kmax, kmin, sc, idx, cnt = oracle_select(case, b)
            nb = kmax.shape[0]
            assert np.array_equal(_to_np(run.kmax)[b].transpose(1, 0, 2)[:nb], kmax)
            assert np.array_equal(_to_np(run.kmin)[b].transpose(1, 0, 2)[:nb], kmin)
            np.testing.assert_allclose(run.scores.cpu().numpy()[b][:, :nb], sc, rtol=2e-5, atol=2e-5)
            got_idx, got_cnt = run.sel_idx.cpu().numpy()[b], run.sel_count.cpu().numpy()[b]
            check_selection(got_idx, got_cnt, idx, cnt, sc, case["ns"], case["nr"], case["k_blocks"], tag)
            sel.append((got_idx, got_cnt))     # attention is judged on the list it was given
        _check_attn(run, case, sel, tag + " " + layout)
        run.out.zero_()
        run.refresh(stale=0)
        torch.cuda.synchronize()
        _check_attn(run, case, None, tag + " full " + layout)


@pytest.mark.parametrize("over,tag", [
    (dict(ctx=[36000], B=64, M=100, tree="uniform"), "G=4, two row tiles, ragged tail"),
    (dict(ctx=[33333, 40000], B=16, M=24, rho=[0.1, 0.1]), "G=4, block 16 (chunks cross blocks), batch of 2"),
    (dict(ctx=[40960, 70], B=64, M=60, rho=[0.1, 0.1]), "G=4, batch with a short sequence (splits without tokens)"),
    (dict(ctx=[34816], B=64, M=30, Hq=10, Hkv=2), "G=5"),
    (dict(ctx=[35000], B=16, M=70, Hq=10, Hkv=2, tree="uniform"), "G=5, two row tiles, block 16"),
    (dict(ctx=[40000], B=64, M=9, Hq=2, Hkv=2), "G=1"),
    (dict(ctx=[33000], B=64, M=40, Hq=4, Hkv=2), "G=2, four wavefronts"),
    (dict(ctx=[36864], B=64, M=60, Hq=16, Hkv=2), "G=8, two workgroups of eight"),
    (dict(ctx=[34000], B=16, M=50, Hq=6, Hkv=2, tree="uniform"), "G=3, six wavefronts, block 16"),
    (dict(ctx=[35840, 33000], B=64, M=60, Hq=10, Hkv=2, rho=[0.1, 0.1]), "G=5, ten row blocks: one workgroup of ten wavefronts, batch of 2"),
    (dict(ctx=[34567], B=16, M=60, Hq=10, Hkv=2, tree="uniform"), "G=5, ten wavefronts, block 16"),
    (dict(ctx=[36000], B=64, M=70, Hq=6, Hkv=2, tree="uniform"), "G=3, nine row blocks: ten wavefronts, one idle"),
    (dict(ctx=[40960, 36000, 30000, 22222, 15000, 9000, 3000, 64], B=64, M=40, rho=[0.1] * 8),
     "G=4, eight wavefronts, ragged batch of 8: workgroups with 0 .. 30 chunks (every remainder of the four-chunk period)"),
    (dict(ctx=[33000, 21000, 9500, 2000, 100], B=64, M=40, Hq=10, Hkv=2, rho=[0.1] * 5),
     "G=5, ten wavefronts, ragged batch of 5"),
])
def test_long_ranges_take_the_group_kernel(gpu_lib, over, tag):
    """Full verification over tens of thousands of tokens at small head counts: each wavefront
    gets eight or more chunks, which selects the kernel that serves all query heads of a KV head
    from one workgroup: 8 wavefronts at G = 4, 6 (one idle) at G = 5 and 32 nodes, 10 at G = 5 and 60 nodes, two
    workgroups for more row blocks, 2 (one idle) at G = 1; head-major (256-byte row stride) and token-major layouts."""
    say("case", tag)
    cfg = dict(SMALL); cfg.update(over)
    case = workloads.to_device(workloads.make_case(cfg, seed=17), "cuda")
    for layout in ("bhtd", "bthd"):
        run = GpuRun(gpu_lib, case, layout=layout)
        run.refresh(stale=0)
        torch.cuda.synchronize()
        _check_attn(run, case, None, tag + " full " + layout)
        sel = [(run.sel_idx.cpu().numpy()[b], run.sel_count.cpu().numpy()[b]) for b in range(case["batch"])]
        run.out.zero_()
        run.attend()
        torch.cuda.synchronize()
        _check_attn(run, case, sel, tag + " partial " + layout)


@pytest.mark.parametrize("dtype,D", [("f32", 64), ("f32", 128), ("bf16", 64)])
@pytest.mark.parametrize("M,ctx,splits", [(128, [1000], 4), (75, [1000], 7), (128, [1000, 900], 2)])
def test_few_splits_on_the_vector_alu_path(gpu_lib, dtype, D, M, ctx, splits):
    """fp32 and head dim 64 take the vector-ALU attention kernel, whose split count falls with the
    number of query rows: 7, 4 and 2 splits here, so that the merge of the partials runs in each
    of its register layouts (8, 4 and 2 partials per round) for these element types too (the
    other cases of this file give them 13 splits or more)."""
    say("case", dtype, D, M, ctx, "splits", splits)
    cfg = dict(SMALL)
    cfg.update(dtype=dtype, D=D, M=M, ctx=ctx, rho=[0.1] * len(ctx), tree="uniform")
    case = workloads.to_device(workloads.make_case(cfg, seed=23), "cuda")
    run = GpuRun(gpu_lib, case)
    # the workspace is sized by the split count: 64 KiB of arrival words + partial O + (m, l) pairs (one slot
    # more than splits) + scores, each rounded up to 256 bytes
    up = lambda x: (x + 255) & ~255
    rows = case["batch"] * case["Hq"] * M
    want = 65536 + up(rows * (splits + 1) * D * 4) + up(rows * (splits + 1) * 8) + \
        up(case["batch"] * case["Hkv"] * case["max_blocks"] * 4)
    assert run.ws.numel() == want, "the planner no longer gives %d splits here" % splits
    run.refresh(stale=0)
    torch.cuda.synchronize()
    _check_attn(run, case, None, "full")
    sel = [(run.sel_idx.cpu().numpy()[b], run.sel_count.cpu().numpy()[b]) for b in range(case["batch"])]
    run.out.zero_()
    run.attend()
    torch.cuda.synchronize()
    _check_attn(run, case, sel, "partial")


@pytest.mark.parametrize("reduce,last_node", [("max", 0), ("last", 0), ("last", 5), ("mean", 0)])
def test_reducers(gpu_lib, reduce, last_node):
    say("reducer", reduce, last_node)
    case = workloads.to_device(workloads.make_case(SMALL, seed=21), "cuda")
    run = GpuRun(gpu_lib, case, reduce=reduce, last_node=last_node)
    run.summarize(); run.select()
    torch.cuda.synchronize()
    o, kmax, kmin, sc, idx, cnt = oracle_select(case, 0, reduce, last_node)
    np.testing.assert_allclose(run.scores.cpu().numpy()[0], sc, rtol=2e-5, atol=2e-5)
    check_selection(run.sel_idx.cpu().numpy()[0], run.sel_count.cpu().numpy()[0], idx, cnt, sc,
                    case["ns"], case["nr"], case["k_blocks"], reduce)


@pytest.mark.parametrize("over,tag", [
    (dict(), "bf16 D=128 (matrix-core scorer)"),
    (dict(dtype="f32", D=64), "f32 D=64 (vector-ALU scorer)"),
    (dict(ctx=[4000], B=64, M=60, k=20), "bf16, 240 query rows over several wavefronts"),
])
@pytest.mark.parametrize("reduce", ["mean", "max"])
def test_channel_bound_scores(gpu_lib, over, tag, reduce):
    """The channel-wise bound as block score (a comparison variant): scores against the oracle's
    per-channel definition, and the selection that follows from them."""
    say("channel bound", tag, reduce)
    cfg = dict(SMALL); cfg.update(over)
    case = workloads.to_device(workloads.make_case(cfg, seed=23), "cuda")
    run = GpuRun(gpu_lib, case, reduce=reduce, score="channel_bound")
    run.summarize(); run.select()
    torch.cuda.synchronize()
    o, kmax, kmin, sc, idx, cnt = oracle_select(case, 0, reduce, 0, score="channel_bound")
    nb = kmax.shape[0]
    got = run.scores.cpu().numpy()[0][:, :nb]
    np.testing.assert_allclose(got, sc, rtol=2e-5, atol=2e-4)
    sc_eq2 = oracle_select(case, 0, reduce, 0)[3]
    assert np.all(got >= sc_eq2 - 1e-3) and np.any(got > sc_eq2 + 1e-2)   # it is a different, larger score
    check_selection(run.sel_idx.cpu().numpy()[0], run.sel_count.cpu().numpy()[0], idx, cnt, sc,
                    case["ns"], case["nr"], case["k_blocks"], "channel bound " + tag)


def test_selection_ties_and_extremes(gpu_lib):
    """Exact ties (duplicated blocks) must go to the lower index; k = 0, no sink, no
    local window and k larger than the candidates are all legal."""
    cfg = dict(SMALL); cfg.update(ctx=[64 * 16], rho=[0.0])
    case = workloads.to_device(workloads.make_case(cfg, seed=31), "cuda")
    B = case["B"]
    k = case["k"]
    # blocks 10, 20, 30, 40 become copies of block 5, and get a large boost so they all rank first
    src = k[0, :, 5 * B:6 * B].clone() + 1.0
    for i in (5, 10, 20, 30, 40):
        k[0, :, i * B:(i + 1) * B] = src
    for (ns, nr, kb) in [(2, 3, 3), (2, 3, 0), (0, 0, 4), (0, 0, 64), (1, 1, 61), (1, 1, 62), (70, 0, 0), (0, 0, 1)]:
        run = GpuRun(gpu_lib, case, cfg=(ns, nr, kb))
        run.summarize(); run.select()
        torch.cuda.synchronize()
        o, kmax, kmin, sc, idx, cnt = oracle_select(case, 0, cfg=(ns, nr, kb))
        got_idx, got_cnt = run.sel_idx.cpu().numpy()[0], run.sel_count.cpu().numpy()[0]
        say("   ns,nr,k =", (ns, nr, kb), "kept", got_idx[0, :got_cnt[0]].tolist()[:12])
        # identical blocks give bit-identical GPU scores
        gs = run.scores.cpu().numpy()[0]
        assert (gs[:, [10, 20, 30, 40]] == gs[:, [5]]).all()
        assert np.array_equal(got_cnt, cnt)
        if kb in (3, 4, 1):   # the tie group decides: must match the oracle exactly
            assert np.array_equal(got_idx, idx), (got_idx, idx)
        else:
            check_selection(got_idx, got_cnt, idx, cnt, sc, ns, nr, kb, "extremes")


def test_selection_over_long_lists(gpu_lib):
    """More than 4096 blocks per head takes the general radix-select kernel (the lists up to
    4096 blocks that the other tests use take the register-resident one): same rule, same
    answer, including an exact tie at the threshold."""
    cfg = dict(SMALL); cfg.update(ctx=[4 * 4300], B=4, M=8, rho=[0.0], name="long_list")
    case = workloads.to_device(workloads.make_case(cfg, seed=5), "cuda")
    B = case["B"]
    k = case["k"]
    src = k[0, :, 7 * B:8 * B].clone() + 1.0
    for i in (7, 1000, 2500, 4200):
        k[0, :, i * B:(i + 1) * B] = src
    for (ns, nr, kb) in [(1, 2, 3), (4, 4, 300), (0, 0, 1)]:
        run = GpuRun(gpu_lib, case, cfg=(ns, nr, kb))
        run.summarize(); run.select()
        torch.cuda.synchronize()
        o, kmax, kmin, sc, idx, cnt = oracle_select(case, 0, cfg=(ns, nr, kb))
        got_idx, got_cnt = run.sel_idx.cpu().numpy()[0], run.sel_count.cpu().numpy()[0]
        say("   4300 blocks, ns,nr,k =", (ns, nr, kb), "kept", got_idx[0, :got_cnt[0]].tolist()[:8])
        assert np.array_equal(got_cnt, cnt)
        if kb in (3, 1):   # the tie group decides: must match the oracle exactly
            assert np.array_equal(got_idx, idx), (got_idx, idx)
        else:
            check_selection(got_idx, got_cnt, idx, cnt, sc, ns, nr, kb, "long list")


def test_attention_list_semantics(gpu_lib):
    """Order of the list is irrelevant, entries past sel_count / negative / out of
    range are ignored, an empty list leaves only the draft segment."""
    case = workloads.to_device(workloads.make_case(SMALL, seed=41), "cuda")
    run = GpuRun(gpu_lib, case)
    nb = 63
    idx = torch.tensor([[[5, 1, 62, 17, 9, -1, 200, 3], [0, 62, 61, 2, 8, 8, 8, 8]]], dtype=torch.int32, device="cuda")
    cnt = torch.tensor([[7, 4]], dtype=torch.int32, device="cuda")
    run.attend(idx, cnt)
    torch.cuda.synchronize()
    # head 0: -1 and 200 are skipped, the 8th entry (3) lies past sel_count = 7
    ref_idx = np.array([[1, 5, 9, 17, 62, -1, -1, -1], [0, 2, 61, 62, -1, -1, -1, -1]], np.int32)
    _check_attn(run, case, [(ref_idx, np.array([5, 4], np.int32))], "list semantics")
    # sorted list gives the same numbers as the shuffled one up to rounding order
    a = run.out.float().clone()
    run.attend(torch.from_numpy(ref_idx)[None].cuda(), torch.tensor([[5, 4]], dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    assert (run.out.float() - a).abs().max() <= 2e-2
    # empty list
    run.attend(idx, torch.zeros_like(cnt))
    torch.cuda.synchronize()
    _check_attn(run, case, [(ref_idx, np.array([0, 0], np.int32))], "empty list")


def test_incremental_summaries_and_stale_refresh(gpu_lib):
    case = workloads.to_device(workloads.make_case(SMALL, seed=51), "cuda")
    run = GpuRun(gpu_lib, case)
    run.summarize(0, 40)
    torch.cuda.synchronize()
    o, kmax, kmin, sc, idx, cnt = oracle_select(case, 0)
    got = _to_np(run.kmax)[0].transpose(1, 0, 2)
    assert np.array_equal(got[:40], kmax[:40]) and (got[40:] == 0).all()
    run.refresh(stale=40)      # recomputes only blocks 40..: the result must now be complete
    torch.cuda.synchronize()
    assert np.array_equal(_to_np(run.kmax)[0].transpose(1, 0, 2), kmax)
    assert np.array_equal(_to_np(run.kmin)[0].transpose(1, 0, 2), kmin)
    check_selection(run.sel_idx.cpu().numpy()[0], run.sel_count.cpu().numpy()[0], idx, cnt, sc,
                    case["ns"], case["nr"], case["k_blocks"], "stale refresh")
    _check_attn(run, case, None, "stale refresh full")


def test_runs_on_a_side_stream_and_is_deterministic(gpu_lib):
    case = workloads.to_device(workloads.make_case(SMALL, seed=61), "cuda")
    run = GpuRun(gpu_lib, case)
    st = torch.cuda.Stream()
    outs = []
    for _ in range(2):
        st.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(st):
            run.out.zero_()
            run.summarize(); run.select(); run.attend()
        st.synchronize()
        outs.append((run.out.clone(), run.sel_idx.clone(), run.lse.clone()))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1]) and torch.equal(outs[0][2], outs[1][2])
    o, kmax, kmin, sc, idx, cnt = oracle_select(case, 0)
    _check_attn(run, case, [(run.sel_idx.cpu().numpy()[0], run.sel_count.cpu().numpy()[0])], "side stream")


@pytest.mark.parametrize("name,seed,n_key,Mq", [("llama8b_16k", 3, 16, 60), ("llama8b_16k", 3, 20, 100),
                                                ("tiny_f32", 2, 5, 16), ("tiny_f32", 2, 1, 16)])
def test_key_only_nodes(gpu_lib, name, seed, n_key, Mq):
    """Section 3.2 (the buffer) on a partial step: the partially verified tokens are a chain of n_key nodes
    in front of the candidates' tree that are attended but have no query rows.  Attention, scores (all
    three reducers count query rows only) and lists against the oracle; full verification too."""
    sp = gpu_lib
    base = workloads.make_case(name, seed=seed, M=Mq)
    gen = torch.Generator().manual_seed(7 + n_key)
    dt = base["q"].dtype
    pk = torch.randn((1, n_key, base["Hkv"], base["D"]), generator=gen).to(dt)
    pv = torch.randn((1, n_key, base["Hkv"], base["D"]), generator=gen).to(dt)
    ext = np.array([oracle.extend_parents(base["parent"][0].tolist(), n_key)], dtype=np.int32)
    case = dict(base)
    case["kd"], case["vd"] = torch.cat([pk, base["kd"]], 1), torch.cat([pv, base["vd"]], 1)
    case["parent"] = torch.from_numpy(ext)
    case = workloads.to_device(case, "cuda")
    for reduce in ("mean", "max", "last"):
        run = GpuRun(sp, case, reduce=reduce, last_node=n_key + 2)
        assert run.tree.n_key_only == n_key and run.tree.Mq == Mq
        run.summarize(); run.select(); run.attend()
        torch.cuda.synchronize()
        o = workloads.oracle_views(case, 0)
        kmax, kmin = oracle.block_summarize(o["K"], case["B"])
        sc = oracle.block_scores(o["Q"], kmax, kmin, reduce, 2)          # the oracle's rows are the query nodes
        np.testing.assert_allclose(run.scores.cpu().numpy()[0], sc, rtol=2e-5, atol=2e-5)
        idx, cnt = oracle.select_blocks(sc, case["ns"], case["nr"], case["k_blocks"])
        check_selection(run.sel_idx.cpu().numpy()[0], run.sel_count.cpu().numpy()[0], idx, cnt, sc,
                        case["ns"], case["nr"], case["k_blocks"], "%s key-only %s" % (name, reduce))
        gi, gc = run.sel_idx.cpu().numpy()[0], run.sel_count.cpu().numpy()[0]
        O, LSE, _ = oracle.tree_attention(o["Q"], o["K"], o["V"], o["Kd"], o["Vd"], o["parent"], case["B"], gi, gc,
                                          n_key_only=n_key)
        err = np.abs(_to_np(run.out)[0] - O).max()
        say("   %s, %d key-only + %d query nodes, %s: attention max-abs err %.3g" % (name, n_key, Mq, reduce, err))
        assert err <= ATOL[case["dtype"]]
        np.testing.assert_allclose(_to_np(run.lse)[0], LSE, atol=2e-5 if case["dtype"] == "f32" else 2e-3, rtol=1e-5)
    run.out.zero_()
    run.attend(None, None)   # every block
    torch.cuda.synchronize()
    O, LSE, _ = oracle.tree_attention(o["Q"], o["K"], o["V"], o["Kd"], o["Vd"], o["parent"], case["B"], n_key_only=n_key)
    assert np.abs(_to_np(run.out)[0] - O).max() <= ATOL[case["dtype"]]


@pytest.mark.parametrize("over,n_key,tag", [
    (dict(ctx=[1000]), 33, "two chunks of pending tokens, the second with one token; block 16 (chunks cross blocks)"),
    (dict(ctx=[2048], B=64, M=60, Hq=8, Hkv=2), 64, "two full chunks, 64-token blocks"),
    (dict(ctx=[1500, 70], B=32, rho=[0.1, 0.1]), 7, "batch of two, one shorter than a block row"),
    (dict(ctx=[36000], B=64, M=60, Hq=8, Hkv=2), 20, "long context: the group kernel, eight wavefronts"),
    (dict(ctx=[35840, 33000], B=64, M=60, Hq=10, Hkv=2, rho=[0.1, 0.1]), 17, "group kernel, ten wavefronts, batch of two"),
    (dict(ctx=[34567], B=16, M=40, Hq=4, Hkv=2), 40, "group kernel, block 16, four wavefronts"),
    (dict(ctx=[3], B=16, M=30), 12, "three cache tokens"),
    (dict(ctx=[1200], dtype="f32", D=64), 9, "f32, D = 64: the vector-ALU kernel leaves them to the combine"),
])
def test_pending_tokens_go_with_the_cache_tokens(gpu_lib, over, n_key, tag):
    """The matrix-core kernels attend the partially verified tokens as extra 32-token chunks behind the cache
    tokens (rows of the draft K / V arrays), the combine kernel stops its root paths at the chain: partial
    attention over the kept lists and attention over every block against the oracle, both layouts."""
    say("case", tag)
    cfg = dict(SMALL); cfg.update(over)
    base = workloads.make_case(cfg, seed=23)
    case = workloads.to_device(with_pending(base, n_key, 100 + n_key), "cuda")
    for layout in ("bhtd", "bthd"):
        run = GpuRun(gpu_lib, case, layout=layout)
        assert run.tree.n_key_only == n_key
        run.summarize(); run.select(); run.attend()
        torch.cuda.synchronize()
        out, lse = _to_np(run.out), _to_np(run.lse)
        for full in (False, True):
            if full:
                run.out.zero_()
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
            say("   %s %s %s: max-abs err %.3g" % (tag, layout, "every block" if full else "kept lists", worst))
            assert worst <= ATOL[case["dtype"]]
