"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py
times (same descriptors, same workspace sizing).  The oracle cannot do 128K x 32
layers in seconds, so: kept-block lists are compared in full (scoring is cheap for
the oracle), attention is compared on a sample of KV heads -- all tree nodes and all
query heads of the sampled KV heads -- which the oracle computes one row at a time."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from helpers import ATOL, GpuRun, check_selection, say, topk_margin

pytestmark = pytest.mark.gpu


def _oracle_scores_and_lists(case, b):
    L = int(case["ctx_len"][b])
    K = case["k"][b, :, :L].permute(1, 0, 2).contiguous().cpu()
    kmax, kmin = oracle.block_summarize(K, case["B"])
    sc = oracle.block_scores(case["q"][b].cpu(), kmax, kmin, "mean")
    idx, cnt = oracle.select_blocks(sc, case["ns"], case["nr"], case["k_blocks"])
    return kmax, kmin, sc, idx, cnt


def _oracle_attention_on_heads(case, b, heads, sel=None):
    """Oracle attention restricted to KV heads `heads` (and their query heads).
    sel = (idx, cnt) numpy of the full head set, or None for every block."""
    G, B = case["G"], case["B"]
    L = int(case["ctx_len"][b])
    qh = [g * G + x for g in heads for x in range(G)]
    Q = case["q"][b][:, qh].cpu()
    Kd, Vd = case["kd"][b][:, heads].cpu(), case["vd"][b][:, heads].cpu()
    parent = case["parent"][b].cpu().numpy()
    if sel is None:
        K = case["k"][b, heads, :L].permute(1, 0, 2).contiguous().cpu()
        V = case["v"][b, heads, :L].permute(1, 0, 2).contiguous().cpu()
        O, lse, ps = oracle.tree_attention(Q, K, V, Kd, Vd, parent, B)
    else:
        idx, cnt = sel
        n = int(cnt[heads].max())
        assert (cnt[heads] == n).all()
        # hand over only the kept blocks, renumbered 0..n-1 per head (attention does not
        # depend on where a block sits); the last block may be partly filled: keep its length
        blocks = torch.from_numpy(idx[heads][:, :n].astype(np.int64))
        tok = (blocks[:, :, None] * B + torch.arange(B)[None, None]).reshape(len(heads), n * B)
        valid = tok < L
        assert valid.all(), "sampled heads must not keep a partly filled block"
        dev = case["k"].device
        K = torch.stack([case["k"][b, g][tok[i].to(dev)] for i, g in enumerate(heads)], 1).cpu()
        V = torch.stack([case["v"][b, g][tok[i].to(dev)] for i, g in enumerate(heads)], 1).cpu()
        O, lse, ps = oracle.tree_attention(Q, K, V, Kd, Vd, parent, B)
    np.testing.assert_allclose(ps, 1.0, atol=1e-12)
    return qh, O, lse


def _compare(run, case, b, qh, O, lse, tag):
    got = run.out[b].float().cpu().numpy()[:, qh]
    err = np.abs(got - O).max()
    say("   %s: max-abs err %.3g over %d rows" % (tag, err, O.shape[0] * O.shape[1]))
    assert err <= ATOL[case["dtype"]], (tag, err)
    np.testing.assert_allclose(run.lse[b].cpu().numpy()[:, qh], lse, atol=2e-3, rtol=1e-5)


@pytest.mark.parametrize("layer", [0, 15, 31])
def test_llama8b_128k_partial_step(gpu_lib, layer):
    """One layer of the headline workload: refresh to get the lists, then the timed call."""
    say("llama8b_128k layer", layer)
    case = workloads.make_case("llama8b_128k", seed=0, layer=layer, device="cuda")   # as bench.py builds it
    run = GpuRun(gpu_lib, case)
    run.refresh(stale=0)
    torch.cuda.synchronize()
    kmax, kmin, sc, idx, cnt = _oracle_scores_and_lists(case, 0)
    assert np.array_equal(run.kmax[0].float().cpu().numpy().transpose(1, 0, 2), kmax)
    np.testing.assert_allclose(run.scores[0].cpu().numpy(), sc, rtol=2e-5, atol=2e-5)
    margin = topk_margin(sc, case["ns"], case["nr"], case["k_blocks"])
    say("   top-k margins", np.array2string(margin, precision=4))
    got_idx, got_cnt = run.sel_idx[0].cpu().numpy(), run.sel_count[0].cpu().numpy()
    check_selection(got_idx, got_cnt, idx, cnt, sc, case["ns"], case["nr"], case["k_blocks"], "128k lists")
    # inputs and kernels are deterministic: at the graded size the lists are pinned bit for bit
    # (also where a margin is below the near-tie band that the random-shape tests allow)
    assert np.array_equal(got_idx, idx) and np.array_equal(got_cnt, cnt), "kept lists differ from the oracle's"
    if layer == 0:
        # the full verification itself at 128K (the launch configuration bench.py times for the refresh)
        qh, O, lse = _oracle_attention_on_heads(case, 0, [6])
        _compare(run, case, 0, qh, O, lse, "full verification at 128K, KV head 6")
    run.out.zero_()
    run.attend()
    torch.cuda.synchronize()
    heads = [layer % 8, (layer + 3) % 8]
    qh, O, lse = _oracle_attention_on_heads(case, 0, heads, (got_idx, got_cnt))
    _compare(run, case, 0, qh, O, lse, "partial, KV heads %s" % heads)


def test_qwen8b_full_verify_refresh_64k(gpu_lib):
    say("qwen8b_refresh_64k")
    case = workloads.make_case("qwen8b_refresh_64k", seed=0, device="cuda")
    run = GpuRun(gpu_lib, case)
    run.refresh(stale=0)
    torch.cuda.synchronize()
    kmax, kmin, sc, idx, cnt = _oracle_scores_and_lists(case, 0)
    assert np.array_equal(run.kmin[0].float().cpu().numpy().transpose(1, 0, 2), kmin)
    got_idx, got_cnt = run.sel_idx[0].cpu().numpy(), run.sel_count[0].cpu().numpy()
    say("   top-k margins", np.array2string(topk_margin(sc, case["ns"], case["nr"], case["k_blocks"]), precision=4))
    check_selection(got_idx, got_cnt, idx, cnt, sc, case["ns"], case["nr"], case["k_blocks"], "64k refresh lists")
    assert np.array_equal(got_idx, idx) and np.array_equal(got_cnt, cnt), "kept lists differ from the oracle's"
    qh, O, lse = _oracle_attention_on_heads(case, 0, [5])
    _compare(run, case, 0, qh, O, lse, "full verification, KV head 5")


def test_qwen14b_ragged_batch(gpu_lib):
    say("qwen14b_batch4")
    case = workloads.make_case("qwen14b_batch4", seed=0, device="cuda")
    run = GpuRun(gpu_lib, case)
    run.summarize(); run.select()
    torch.cuda.synchronize()
    lists = []
    for b in range(case["batch"]):
        kmax, kmin, sc, idx, cnt = _oracle_scores_and_lists(case, b)
        got_idx, got_cnt = run.sel_idx[b].cpu().numpy(), run.sel_count[b].cpu().numpy()
        check_selection(got_idx, got_cnt, idx, cnt, sc, case["ns"], case["nr"], case["k_blocks"], "seq %d" % b)
        say("   seq %d (L=%d): min margin %.4f" % (
            b, int(case["ctx_len"][b]), topk_margin(sc, case["ns"], case["nr"], case["k_blocks"]).min()))
        assert np.array_equal(got_idx, idx) and np.array_equal(got_cnt, cnt), "seq %d: kept lists differ from the oracle's" % b
        lists.append((got_idx, got_cnt))
    run.attend()
    torch.cuda.synchronize()
    for b in range(case["batch"]):
        qh, O, lse = _oracle_attention_on_heads(case, b, [(2 * b + 1) % 8], lists[b])
        _compare(run, case, b, qh, O, lse, "seq %d partial" % b)
    # full verification of the shortest and of the longest sequence (G = 5: one workgroup of ten
    # wavefronts per KV head and split, many splits because the lengths differ)
    run.refresh(stale=-1)
    torch.cuda.synchronize()
    qh, O, lse = _oracle_attention_on_heads(case, 0, [3])
    _compare(run, case, 0, qh, O, lse, "seq 0 full")
    qh, O, lse = _oracle_attention_on_heads(case, 3, [6])
    _compare(run, case, 3, qh, O, lse, "seq 3 (the longest) full")


def test_paper_default_geometry(gpu_lib):
    """Block 16, 32 sink + 128 local tokens, 4K budget (Appendix D of the paper) at 60K context."""
    say("paper_default_4k")
    case = workloads.make_case("paper_default_4k", seed=0, device="cuda")
    run = GpuRun(gpu_lib, case)
    run.refresh(stale=0)
    torch.cuda.synchronize()
    kmax, kmin, sc, idx, cnt = _oracle_scores_and_lists(case, 0)
    got_idx, got_cnt = run.sel_idx[0].cpu().numpy(), run.sel_count[0].cpu().numpy()
    check_selection(got_idx, got_cnt, idx, cnt, sc, case["ns"], case["nr"], case["k_blocks"], "paper default")
    assert np.array_equal(got_idx, idx) and np.array_equal(got_cnt, cnt), "kept lists differ from the oracle's"
    run.attend()
    torch.cuda.synchronize()
    qh, O, lse = _oracle_attention_on_heads(case, 0, [1, 6], (got_idx, got_cnt))
    _compare(run, case, 0, qh, O, lse, "partial, block 16")


@pytest.mark.parametrize("budget", [512, 2048, 8192])
def test_paper_budgets(gpu_lib, budget):
    """The partial-cache budgets of Table 1 / Figure 5 (512, 2K, 8K tokens) in the paper's geometry
    (Appendix D: 16-token blocks, 32 sink and 128 local tokens) at 60K context: the retrieval
    part is k = (budget - 32 - 128) / 16 blocks."""
    case = workloads.make_case("paper_default_4k", seed=1, device="cuda")
    ns, nr = 2, 8
    kb = (budget - ns * 16 - nr * 16) // 16
    run = GpuRun(gpu_lib, case, cfg=(ns, nr, kb))
    run.summarize(); run.select()
    torch.cuda.synchronize()
    L = int(case["ctx_len"][0])
    K = case["k"][0, :, :L].permute(1, 0, 2).contiguous().cpu()
    kmax, kmin = oracle.block_summarize(K, case["B"])
    sc = oracle.block_scores(case["q"][0].cpu(), kmax, kmin, "mean")
    idx, cnt = oracle.select_blocks(sc, ns, nr, kb)
    got_idx, got_cnt = run.sel_idx[0].cpu().numpy(), run.sel_count[0].cpu().numpy()
    exact = check_selection(got_idx, got_cnt, idx, cnt, sc, ns, nr, kb, "budget %d" % budget)
    assert np.array_equal(got_idx, idx) and np.array_equal(got_cnt, cnt), "kept lists differ from the oracle's"
    assert (got_cnt == ns + nr + kb).all()
    run.attend()
    torch.cuda.synchronize()
    qh, O, lse = _oracle_attention_on_heads(case, 0, [2, 5], (got_idx, got_cnt))
    _compare(run, case, 0, qh, O, lse, "budget %d (k = %d blocks, lists bit-exact: %s)" % (budget, kb, exact))
