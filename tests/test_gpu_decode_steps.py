"""GPU parity of the verification modes and the buffer (Section 3.3, Algorithm 1): a
synthetic multi-step decode.  Every step picks the mode with the library's SelectMode, runs
the attention the mode prescribes on the device state (partial over the kept blocks, or
full + refresh, with the partially verified tokens as the chain prefix of the tree), accepts a
seeded random root path, and commits it.  The fp64 oracle runs the same steps on its own
copy of the state.  Bars: modes, lengths, cache rows, buffer rows, summaries and kept
lists bit-exact (lists under the near-tie margin rule); attention outputs max-abs <= 2e-2
(bf16) / 1e-5 (fp32)."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from helpers import ATOL, check_selection, say

pytestmark = pytest.mark.gpu


def _f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("dtype,D,B,Hq,Hkv,M,L0,nbm", [("bf16", 128, 16, 8, 2, 12, 215, 64),
                                                      ("f32", 64, 8, 4, 2, 9, 130, 64),
                                                      ("bf16", 128, 16, 8, 2, 12, 215, 15)])   # the cache fills up
def test_multi_step_decode(gpu_lib, dtype, D, B, Hq, Hkv, M, L0, nbm):
    sp = gpu_lib
    dev = torch.device("cuda")
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    rng = np.random.default_rng(1234 + D)
    gen = torch.Generator().manual_seed(99 + D)
    ns, nr, kb = 2, 3, 9
    budget = (ns + nr + kb) * B                # the partial cache without the buffer
    margin, max_accept = 6, 5
    P = margin + max_accept + 1                # room for the pending tokens
    T = nbm * B                                # capacity in tokens
    extra = (P + max_accept + B - 1) // B + 1  # list entries for the blocks that commits append

    def rnd(*shape):
        return torch.randn(shape, generator=gen).to(tdt)

    # device state
    k, v = torch.zeros((1, Hkv, T, D), dtype=tdt), torch.zeros((1, Hkv, T, D), dtype=tdt)
    k[0, :, :L0], v[0, :, :L0] = rnd(Hkv, L0, D), rnd(Hkv, L0, D)
    k, v = k.to(dev), v.to(dev)
    ctx_len = torch.tensor([L0], dtype=torch.int32, device=dev)
    kv = sp.KV(k, v, ctx_len, B, nbm)
    buf_k = torch.zeros((1, P + M, Hkv, D), dtype=tdt, device=dev)
    buf_v = torch.zeros_like(buf_k)
    n_pending = torch.zeros((1,), dtype=torch.int32, device=dev)
    dropped = torch.full((1, 2), -9, dtype=torch.int32, device=dev)
    kmax = torch.zeros((1, Hkv, nbm, D), dtype=tdt, device=dev)
    kmin = torch.zeros_like(kmax)
    cfg = sp.SelectCfg(ns, nr, kb, "mean", n_extra_slots=extra)
    sel_idx = torch.full((1, Hkv, cfg.n_sel), -1, dtype=torch.int32, device=dev)
    sel_count = torch.zeros((1, Hkv), dtype=torch.int32, device=dev)
    sp.specpv_block_summarize(kv, 0, -1, kmax, kmin)
    # oracle state: K / V [T, Hkv, D] float64 copies of the same numbers
    Ko, Vo = _f64(k[0]).transpose(1, 0, 2).copy(), _f64(v[0]).transpose(1, 0, 2).copy()
    L, pend_k, pend_v, ready = L0, [], [], False
    o_idx = o_cnt = None
    modes, lost = [], 0
    for step in range(16):
        n = len(pend_k)
        mode = sp.specpv_select_mode(budget, margin, L + n, ready, n)
        assert mode == oracle.select_mode(L + n, ready, n, budget, margin)
        modes.append(mode)
        # this step's candidates; the pending tokens are keys only on a partial step (no query rows) and
        # ordinary nodes, with recomputed K/V, on a full verification
        nq = M if mode == sp.MODE_PARTIAL else n + M
        tree = workloads.make_tree(M, "bounded", rng, max_depth=max_accept - 1)
        q, kd, vd = rnd(1, nq, Hq, D).to(dev), rnd(1, M, Hkv, D).to(dev), rnd(1, M, Hkv, D).to(dev)
        buf_k[:, P:], buf_v[:, P:] = kd, vd
        if mode != sp.MODE_PARTIAL and n > 0:
            nk, nv = rnd(1, n, Hkv, D).to(dev), rnd(1, n, Hkv, D).to(dev)
            buf_k[:, P - n:P], buf_v[:, P - n:P] = nk, nv
            pend_k, pend_v = list(_f64(nk[0])), list(_f64(nv[0]))
        ext = sp.specpv_extend_parents(tree.tolist(), n)
        assert ext == oracle.extend_parents(tree.tolist(), n)
        parent = torch.tensor([ext], dtype=torch.int32, device=dev)
        tr = sp.Tree(q, buf_k[:, P - n:], buf_v[:, P - n:], parent)
        assert tr.n_key_only == (n if mode == sp.MODE_PARTIAL else 0)
        out = torch.zeros_like(q)
        lse = torch.zeros((1, nq, Hq), dtype=torch.float32, device=dev)
        ws = torch.zeros((sp.specpv_workspace_bytes(kv, tr, cfg),), dtype=torch.uint8, device=dev)
        Qo = _f64(q[0])
        Kd_o = np.stack(pend_k + list(_f64(kd[0])))
        Vd_o = np.stack(pend_v + list(_f64(vd[0])))
        if mode == sp.MODE_PARTIAL:
            sp.specpv_partial_verify_attn(kv, tr, sel_idx, sel_count, out, lse, ws)
            O, LSE, _ = oracle.tree_attention(Qo, Ko[:L], Vo[:L], Kd_o, Vd_o, np.array(ext, np.int32), B, o_idx, o_cnt,
                                              n_key_only=n)
        elif L + n <= budget:
            sp.specpv_partial_verify_attn(kv, tr, None, None, out, lse, ws)      # plain full verification
            O, LSE, _ = oracle.tree_attention(Qo, Ko[:L], Vo[:L], Kd_o, Vd_o, np.array(ext, np.int32), B)
        else:
            # full verification that (re)builds the partial cache with this pass's queries
            sp.specpv_full_verify_refresh(kv, tr, kmax, kmin, -1, cfg, out, lse, sel_idx, sel_count, None, ws)
            O, LSE, o_idx, o_cnt, sc = oracle.full_verify_refresh(Qo, Ko[:L], Vo[:L], Kd_o, Vd_o,
                                                                  np.array(ext, np.int32), B, ns, nr, kb)
            torch.cuda.synchronize()
            got_idx, got_cnt = sel_idx.cpu().numpy()[0], sel_count.cpu().numpy()[0]
            assert (got_idx[:, ns + nr + kb:] == -1).all(), "the free entries of a fresh list row are -1"
            check_selection(got_idx[:, :ns + nr + kb], got_cnt, o_idx, o_cnt, sc, ns, nr, kb, "step %d" % step)
            o_idx, o_cnt = got_idx.copy(), got_cnt.copy()   # continue on the device's lists
            ready = True
        torch.cuda.synchronize()
        err = np.abs(_f64(out[0]) - O).max()
        assert err <= ATOL[dtype], (step, mode, err)
        np.testing.assert_allclose(lse[0].cpu().numpy(), LSE, atol=2e-3, rtol=1e-5)
        # a seeded random accepted root path
        path, node = [0], 0
        want = int(rng.integers(1, max_accept + 1))
        while len(path) < want:
            kids = [j for j in range(M) if tree[j] == node]
            if not kids:
                break
            node = kids[int(rng.integers(0, len(kids)))]
            path.append(node)
        acc = torch.full((1, max_accept), -1, dtype=torch.int32)
        acc[0, :len(path)] = torch.tensor(path, dtype=torch.int32)
        n_acc = torch.tensor([len(path)], dtype=torch.int32, device=dev)
        L_before = L
        sp.specpv_commit_accepted(kv, buf_k, buf_v, P, M, n_pending, acc.to(dev), n_acc, mode, kmax, kmin, ws,
                                  sel_idx=sel_idx, sel_count=sel_count, dropped=dropped)
        want_drop = oracle.commit_dropped(L, len(pend_k), len(path), mode, T, P)
        L, pend_k, pend_v = oracle.commit_accepted(Ko, Vo, L, pend_k, pend_v, _f64(kd[0]), _f64(vd[0]), path, mode, T, P)
        torch.cuda.synchronize()
        assert int(ctx_len[0]) == L and int(n_pending[0]) == len(pend_k), (step, mode)
        assert dropped[0].tolist() == [want_drop, 0], (step, dropped.tolist(), want_drop)
        lost += want_drop
        if o_idx is not None and mode != sp.MODE_PARTIAL:
            # Section 3.3: the committed tokens stay in the partial cache -- the lists follow the length
            o_idx, o_cnt, miss = oracle.extend_lists(o_idx, o_cnt, L_before, L, B)
            assert not miss.any()
            assert np.array_equal(sel_idx.cpu().numpy()[0], o_idx) and np.array_equal(sel_count.cpu().numpy()[0], o_cnt), \
                (step, "kept lists after the commit")
        kd_all, vd_all = _f64(k[0]).transpose(1, 0, 2), _f64(v[0]).transpose(1, 0, 2)
        assert np.array_equal(kd_all[:L], Ko[:L]) and np.array_equal(vd_all[:L], Vo[:L]), (step, "cache rows")
        assert not kd_all[L:].any() and not vd_all[L:].any(), (step, "rows beyond the committed length")
        if pend_k:
            m = len(pend_k)
            assert np.array_equal(_f64(buf_k[0, P - m:P]), np.stack(pend_k)), (step, "pending K rows")
            assert np.array_equal(_f64(buf_v[0, P - m:P]), np.stack(pend_v)), (step, "pending V rows")
        nb = (L + B - 1) // B
        omax, omin = oracle.block_summarize(Ko[:L], B)
        assert np.array_equal(_f64(kmax[0, :, :nb]), omax.transpose(1, 0, 2)), (step, "kmax")
        assert np.array_equal(_f64(kmin[0, :, :nb]), omin.transpose(1, 0, 2)), (step, "kmin")
        say("   step %2d mode %s: %d pending before, accepted %d, L %d -> %d, dropped %d, attention err %.3g"
            % (step, ["FULL", "PARTIAL", "REFRESH"][mode], n, len(path), L_before, L, want_drop, err))
    assert sp.MODE_PARTIAL in modes and sp.MODE_REFRESH in modes and modes[0] == sp.MODE_FULL
    if nbm * B < L0 + 40:
        assert L == T and lost > 0, "this case is meant to fill the cache"


def test_list_rows_that_are_too_short_are_reported(gpu_lib):
    """A commit to the cache with list rows that have no free entry: the blocks are not listed, nothing is
    written out of bounds, and dropped[b, 1] says how many blocks found no room (bit-exact vs the oracle)."""
    sp = gpu_lib
    dev = torch.device("cuda")
    Hkv, D, B, nbm, P, M = 2, 64, 8, 16, 12, 6
    k = torch.zeros((1, Hkv, nbm * B, D), device=dev)
    v = torch.zeros_like(k)
    L0 = 43
    ctx_len = torch.tensor([L0], dtype=torch.int32, device=dev)
    kv = sp.KV(k, v, ctx_len, B, nbm)
    buf_k = torch.randn((1, P + M, Hkv, D), device=dev)
    buf_v = torch.randn_like(buf_k)
    n_pending = torch.tensor([9], dtype=torch.int32, device=dev)
    acc = torch.tensor([[0, 2, 3, 5]], dtype=torch.int32, device=dev)
    n_acc = torch.tensor([4], dtype=torch.int32, device=dev)
    rows = np.array([[0, 3, 5, -1], [0, 1, 4, 5]], np.int32)     # head 0 has one free entry, head 1 none
    cnts = np.array([3, 4], np.int32)
    big = torch.full((1, Hkv + 1, 4), 77, dtype=torch.int32, device=dev)   # one guard row behind the lists
    big[0, :Hkv] = torch.from_numpy(rows).to(dev)
    sel_idx = big[:, :Hkv]
    sel_count = torch.from_numpy(cnts[None].copy()).to(dev)
    dropped = torch.zeros((1, 2), dtype=torch.int32, device=dev)
    ws = torch.zeros((sp.specpv_workspace_bytes(kv),), dtype=torch.uint8, device=dev)
    sp.specpv_commit_accepted(kv, buf_k, buf_v, P, M, n_pending, acc, n_acc, sp.MODE_REFRESH, None, None, ws,
                              sel_idx=sel_idx, sel_count=sel_count, dropped=dropped)
    torch.cuda.synchronize()
    L = L0 + 13
    assert int(ctx_len[0]) == L
    o_idx, o_cnt, miss = oracle.extend_lists(rows, cnts, L0, L, B)        # blocks 5 and 6 receive tokens
    assert np.array_equal(sel_idx.cpu().numpy()[0], o_idx) and np.array_equal(sel_count.cpu().numpy()[0], o_cnt)
    assert dropped[0].tolist() == [0, int(miss.max())] and miss.max() == 1
    assert (big[0, Hkv] == 77).all()


@pytest.mark.parametrize("name,seed", [("llama8b_16k", 3), ("paper_default_4k", 0)])
def test_gathered_partial_cache(gpu_lib, name, seed):
    """Section 3.2's physically contiguous partial cache: the gather is bit-exact against the
    oracle's, and attention over the gathered segment (no list) gives what attention over the
    lists gives (same kernel, same token order) and what the oracle gives."""
    from helpers import GpuRun
    sp = gpu_lib
    case = workloads.to_device(workloads.make_case(name, seed=seed), "cuda")
    run = GpuRun(sp, case)
    run.refresh(stale=0)
    run.attend()
    torch.cuda.synchronize()
    B, Hkv, D, n_sel = case["B"], case["Hkv"], case["D"], run.cfg.n_sel
    dev = case["q"].device
    gk = torch.full((1, Hkv, n_sel * B, D), 7.0, dtype=case["q"].dtype, device=dev)
    gv = torch.full_like(gk, 7.0)
    glen = torch.full((1,), -5, dtype=torch.int32, device=dev)
    sp.specpv_gather_blocks(run.kv, run.sel_idx, run.sel_count, gk, gv, glen)
    torch.cuda.synchronize()
    o = workloads.oracle_views(case, 0)
    idx, cnt = run.sel_idx.cpu().numpy()[0], run.sel_count.cpu().numpy()[0]
    Kg, Vg, rows = oracle.gather_blocks(o["K"], o["V"], B, idx, cnt)
    assert int(glen[0]) == int(rows.max())
    assert np.array_equal(_f64(gk[0]).transpose(1, 0, 2), Kg) and np.array_equal(_f64(gv[0]).transpose(1, 0, 2), Vg)
    # attention over the gathered segment
    kv2 = sp.KV(gk, gv, glen, B, n_sel)
    out2 = torch.zeros_like(run.out)
    lse2 = torch.zeros_like(run.lse)
    ws2 = torch.zeros((sp.specpv_workspace_bytes(kv2, run.tree, run.cfg),), dtype=torch.uint8, device=dev)
    sp.specpv_partial_verify_attn(kv2, run.tree, None, None, out2, lse2, ws2)
    torch.cuda.synchronize()
    d = np.abs(_f64(out2[0]) - _f64(run.out[0])).max()
    say("   %s: gathered vs indexed attention max-abs diff %.3g" % (name, d))
    assert d <= 2e-2 * 0.25
    O, LSE, _ = oracle.tree_attention(o["Q"], o["K"], o["V"], o["Kd"], o["Vd"], o["parent"], B, idx, cnt)
    assert np.abs(_f64(out2[0]) - O).max() <= ATOL[case["dtype"]]


@pytest.mark.parametrize("mode_name", ["partial", "refresh"])
def test_commit_of_all_layers_at_once(gpu_lib, mode_name):
    """specpv_commit_accepted_layers on 34 layers (more than one launch's worth) that share their
    length counters gives, bit for bit, what specpv_commit_accepted gives layer by layer on private
    copies of the counters (which the decode test above checks against the oracle)."""
    sp = gpu_lib
    dev = torch.device("cuda")
    g = torch.Generator(device="cpu").manual_seed(77)
    n_layers, batch, Hkv, D, T, B, P, Mt = 34, 2, 2, 128, 512, 16, 28, 24
    mode = sp.MODE_PARTIAL if mode_name == "partial" else sp.MODE_REFRESH

    def rnd(*shape):
        return torch.randn(shape, generator=g).to(torch.bfloat16).to(dev)
    ks = [rnd(batch, Hkv, T, D) for _ in range(n_layers)]
    vs = [rnd(batch, Hkv, T, D) for _ in range(n_layers)]
    bks = [rnd(batch, P + Mt, Hkv, D) for _ in range(n_layers)]
    bvs = [rnd(batch, P + Mt, Hkv, D) for _ in range(n_layers)]
    ctx0 = torch.tensor([100, 333], dtype=torch.int32, device=dev)
    pend0 = torch.tensor([5, 0], dtype=torch.int32, device=dev)
    accepted = torch.tensor([[0, 2, 5, 9], [1, 3, 0, 0]], dtype=torch.int32, device=dev)
    n_acc = torch.tensor([4, 2], dtype=torch.int32, device=dev)
    max_blocks = T // B
    ws = torch.zeros((1 << 17,), dtype=torch.uint8, device=dev)
    # kept-block lists per layer: [0, l % 3 + 1, the block in front of the last one], five free entries
    lists0 = []
    for l in range(n_layers):
        si = torch.full((batch, Hkv, 8), -1, dtype=torch.int32)
        for b, Lb in enumerate((100, 333)):
            si[b, :, :3] = torch.tensor([0, l % 3 + 1, (Lb - 1) // B - 1], dtype=torch.int32)
        lists0.append((si.to(dev), torch.full((batch, Hkv), 3, dtype=torch.int32, device=dev)))

    # layer by layer, private counters
    ref = []
    for l in range(n_layers):
        k, v, bk, bv = ks[l].clone(), vs[l].clone(), bks[l].clone(), bvs[l].clone()
        ctx, pend = ctx0.clone(), pend0.clone()
        kv = sp.KV(k, v, ctx, B, max_blocks)
        kmax = torch.zeros(kv.summary_shape(), dtype=k.dtype, device=dev); kmin = torch.zeros_like(kmax)
        sp.specpv_block_summarize(kv, 0, -1, kmax, kmin)
        si, sc_ = lists0[l][0].clone(), lists0[l][1].clone()
        drop = torch.full((batch, 2), -1, dtype=torch.int32, device=dev)
        sp.specpv_commit_accepted(kv, bk, bv, P, Mt, pend, accepted, n_acc, mode, kmax, kmin, ws,
                                  sel_idx=si, sel_count=sc_, dropped=drop)
        ref.append((k, v, bk, bv, ctx, pend, kmax, kmin, si, sc_, drop))
    # all layers at once, shared counters
    ctx, pend = ctx0.clone(), pend0.clone()
    k2, v2 = [x.clone() for x in ks], [x.clone() for x in vs]
    bk2, bv2 = [x.clone() for x in bks], [x.clone() for x in bvs]
    kvs = [sp.KV(k2[l], v2[l], ctx, B, max_blocks) for l in range(n_layers)]
    kmaxs, kmins = [], []
    for l in range(n_layers):
        kmax = torch.zeros(kvs[l].summary_shape(), dtype=k2[l].dtype, device=dev); kmin = torch.zeros_like(kmax)
        sp.specpv_block_summarize(kvs[l], 0, -1, kmax, kmin)
        kmaxs.append(kmax); kmins.append(kmin)
    say("commit of", n_layers, "layers,", mode_name)
    si2, sc2 = [x[0].clone() for x in lists0], [x[1].clone() for x in lists0]
    drop2 = torch.full((batch, 2), -1, dtype=torch.int32, device=dev)
    sp.specpv_commit_accepted_layers(kvs, bk2, bv2, P, Mt, pend, accepted, n_acc, mode, kmaxs, kmins, ws,
                                     sel_idxs=si2, sel_counts=sc2, dropped=drop2)
    torch.cuda.synchronize()
    for l in range(n_layers):
        k, v, bk, bv, c1, p1, kmax, kmin, si, sc_, drop = ref[l]
        assert torch.equal(si2[l], si) and torch.equal(sc2[l], sc_), "kept lists, layer %d" % l
        assert torch.equal(drop2, drop) and drop.tolist() == [[0, 0], [0, 0]]
        assert torch.equal(k2[l], k) and torch.equal(v2[l], v), "cache rows, layer %d" % l
        assert torch.equal(bk2[l], bk) and torch.equal(bv2[l], bv), "buffer rows, layer %d" % l
        assert torch.equal(kmaxs[l], kmax) and torch.equal(kmins[l], kmin), "summaries, layer %d" % l
        assert torch.equal(ctx, c1) and torch.equal(pend, p1), "counters"
    if mode_name == "partial":
        assert ctx.tolist() == [100, 333] and pend.tolist() == [9, 2]
        assert all(torch.equal(a, b[0]) for a, b in zip(si2, lists0)), "a partial step leaves the lists alone"
    else:
        assert ctx.tolist() == [109, 335] and pend.tolist() == [0, 0]
        # 100 -> 109 goes to block 6, 333 -> 335 to block 20: neither was listed, both join
        for l in range(n_layers):
            assert si2[l][:, :, 3].tolist() == [[6] * Hkv, [20] * Hkv] and sc2[l].tolist() == [[4] * Hkv] * 2
            assert torch.equal(si2[l][:, :, :3], lists0[l][0][:, :, :3]) and (si2[l][:, :, 4:] == -1).all()
