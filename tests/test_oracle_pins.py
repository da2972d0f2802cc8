"""Pins of the CPU fp64 oracle against what the paper's definitions and plain
mathematics fix: hand-worked examples (tests/golden), closed forms, brute force
on tiny inputs, and reductions to numpy / torch library routines."""
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
import workloads

GOLD = os.path.join(os.path.dirname(__file__), "golden")
rng0 = np.random.default_rng(1234)


def _rand(*shape, rng=None):
    return (rng or rng0).standard_normal(shape)


# ------------------------------------------------------------------ eq. 1
def test_summaries_hand_example():
    g = json.load(open(os.path.join(GOLD, "eq1_eq2_eq3_hand_example.json")))
    kmax, kmin = oracle.block_summarize(np.array(g["K"], float), g["B"])
    assert np.array_equal(kmax, np.array(g["kmax"], float))
    assert np.array_equal(kmin, np.array(g["kmin"], float))


@pytest.mark.parametrize("L,B", [(64, 16), (70, 16), (5, 8), (33, 1)])
def test_summaries_match_numpy_amax_amin(L, B):
    K = _rand(L, 3, 5)
    kmax, kmin = oracle.block_summarize(K, B)
    nb = (L + B - 1) // B
    assert kmax.shape == (nb, 3, 5)
    for i in range(nb):
        blk = K[i * B:min((i + 1) * B, L)]
        assert np.array_equal(kmax[i], blk.max(axis=0))
        assert np.array_equal(kmin[i], blk.min(axis=0))
    if B == 1:
        assert np.array_equal(kmax, K) and np.array_equal(kmin, K)


# ------------------------------------------------------------------ eq. 2, 3
def test_scores_hand_example():
    g = json.load(open(os.path.join(GOLD, "eq1_eq2_eq3_hand_example.json")))
    Q = np.array(g["Q"], float)
    kmax, kmin = np.array(g["kmax"], float), np.array(g["kmin"], float)
    s = oracle.row_scores(Q, kmax, kmin)
    assert np.array_equal(s, np.array(g["row_scores"], float))
    assert np.array_equal(oracle.reduce_scores(s, 2, 2, "mean"), np.array(g["mean"]))
    assert np.array_equal(oracle.reduce_scores(s, 2, 2, "max"), np.array(g["max"]))
    assert np.array_equal(oracle.reduce_scores(s, 2, 2, "last", 0), np.array(g["last_node0"]))
    assert np.array_equal(oracle.reduce_scores(s, 2, 2, "last", 1), np.array(g["last_node1"]))


def test_scores_block_of_one_token_is_plain_dot_product():
    # B = 1: Kmax = Kmin = K, so eq. 2 collapses to q . k (library einsum).
    M, Hq, Hkv, D, L = 5, 6, 2, 7, 11
    G = Hq // Hkv
    Q, K = _rand(M, Hq, D), _rand(L, Hkv, D)
    kmax, kmin = oracle.block_summarize(K, 1)
    s = oracle.row_scores(Q, kmax, kmin)                       # [Hkv, L, M*G]
    ref = np.einsum("jghd,tgd->gtjh", Q.reshape(M, Hkv, G, D), K).reshape(Hkv, L, M * G)
    np.testing.assert_allclose(s, ref, rtol=0, atol=1e-12)


def test_channel_bound_hand_example():
    g = json.load(open(os.path.join(GOLD, "eq1_eq2_eq3_hand_example.json")))
    Q = np.array(g["Q"], float)
    kmax, kmin = np.array(g["kmax"], float), np.array(g["kmin"], float)
    s = oracle.row_scores(Q, kmax, kmin, "channel_bound")
    assert np.array_equal(s, np.array(g["row_scores_channel_bound"], float))
    assert np.array_equal(oracle.reduce_scores(s, 2, 2, "mean"), np.array(g["mean_channel_bound"]))
    assert np.array_equal(oracle.block_scores(Q, kmax, kmin, "mean", 0, "channel_bound"), np.array(g["mean_channel_bound"]))


def test_channel_bound_is_an_upper_bound_and_tight_for_single_tokens():
    # What defines the variant: it bounds q . k_t from above for EVERY token of the block (eq. 2
    # does not), it is never below eq. 2, it equals q . k for blocks of one token, and it is
    # attained when a block's tokens are all alike.
    M, Hq, Hkv, D, L, B = 4, 6, 2, 9, 40, 8
    G = Hq // Hkv
    rng = np.random.default_rng(77)
    Q, K = rng.standard_normal((M, Hq, D)), rng.standard_normal((L, Hkv, D))
    kmax, kmin = oracle.block_summarize(K, B)
    sc = oracle.row_scores(Q, kmax, kmin, "channel_bound")        # [Hkv, nb, M*G]
    s2 = oracle.row_scores(Q, kmax, kmin, "eq2")
    assert np.all(sc >= s2 - 1e-12)
    assert np.any(sc > s2 + 1e-6)
    dots = np.einsum("jghd,tgd->gtjh", Q.reshape(M, Hkv, G, D), K).reshape(Hkv, L, M * G)
    per_block_max = dots.reshape(Hkv, L // B, B, M * G).max(axis=2)
    assert np.all(sc >= per_block_max - 1e-12)
    assert not np.all(s2 >= per_block_max - 1e-12)                # eq. 2 is no such bound
    k1max, k1min = oracle.block_summarize(K, 1)
    np.testing.assert_allclose(oracle.row_scores(Q, k1max, k1min, "channel_bound"), dots, rtol=0, atol=1e-12)
    Kc = np.repeat(K[:5], B, axis=0)                              # 5 blocks of identical tokens
    cmax, cmin = oracle.block_summarize(Kc, B)
    np.testing.assert_allclose(oracle.row_scores(Q, cmax, cmin, "channel_bound"), dots[:, :5], rtol=0, atol=1e-12)


def test_scores_gqa_head_mapping_and_row_order():
    # A query head must only see the summaries of KV head h // G, and row
    # r = j*G + hh.  Make every (node, head) pair and every KV head distinct.
    M, Hq, Hkv, D = 3, 4, 2, 2
    Q = np.zeros((M, Hq, D))
    for j in range(M):
        for h in range(Hq):
            Q[j, h] = [1 + j, 10 * (1 + h)]
    kmax = np.zeros((1, Hkv, D))
    kmin = np.zeros((1, Hkv, D))
    kmax[0, 0], kmin[0, 0] = [1, 0], [1, 0]      # KV head 0 reads coordinate 0
    kmax[0, 1], kmin[0, 1] = [0, 1], [0, 1]      # KV head 1 reads coordinate 1
    s = oracle.row_scores(Q, kmax, kmin)         # [2, 1, 6]
    assert s[0, 0].tolist() == [1, 1, 2, 2, 3, 3]
    assert s[1, 0].tolist() == [30, 40, 30, 40, 30, 40]


def test_scores_invariants():
    M, Hq, Hkv, D, L, B = 6, 8, 2, 16, 96, 8
    Q, K = _rand(M, Hq, D), _rand(L, Hkv, D)
    kmax, kmin = oracle.block_summarize(K, B)
    s = oracle.row_scores(Q, kmax, kmin)
    # symmetric in the two summaries
    assert np.array_equal(s, oracle.row_scores(Q, kmin, kmax))
    # positively homogeneous in q
    np.testing.assert_allclose(oracle.row_scores(2.5 * Q, kmax, kmin), 2.5 * s, rtol=1e-11, atol=1e-12)
    # max over rows >= mean over rows; a constant block scores q . k
    G = Hq // Hkv
    assert (oracle.reduce_scores(s, M, G, "max") >= oracle.reduce_scores(s, M, G, "mean")).all()
    Kc = np.repeat(K[:1], L, axis=0)
    kmx, kmn = oracle.block_summarize(Kc, B)
    sc = oracle.row_scores(Q, kmx, kmn)
    ref = np.einsum("jghd,gd->gjh", Q.reshape(M, Hkv, G, D), K[0]).reshape(Hkv, 1, M * G)
    np.testing.assert_allclose(sc, np.broadcast_to(ref, sc.shape), atol=1e-12)
    # eq. 2 is NOT the channel-wise upper bound: it never exceeds it, and differs
    chan = np.einsum("jghd,igd->gijh", np.maximum(Q, 0).reshape(M, Hkv, G, D), kmax) + \
        np.einsum("jghd,igd->gijh", np.minimum(Q, 0).reshape(M, Hkv, G, D), kmin)
    chan = chan.reshape(Hkv, -1, M * G)
    assert (s <= chan + 1e-12).all() and (s < chan - 1e-6).any()


def test_reduce_matches_numpy():
    s = _rand(3, 10, 4 * 5)
    np.testing.assert_allclose(oracle.reduce_scores(s, 4, 5, "mean"), s.mean(-1), atol=1e-14)
    assert np.array_equal(oracle.reduce_scores(s, 4, 5, "max"), s.max(-1))
    np.testing.assert_allclose(oracle.reduce_scores(s, 4, 5, "last", 2), s[:, :, 10:15].mean(-1), atol=1e-14)


# ------------------------------------------------------------------ selection
def _brute_select(scores, ns, nr, k):
    Hkv, nb = scores.shape
    out = []
    for g in range(Hkv):
        if nb <= ns + k + nr:
            out.append(list(range(nb)))
            continue
        cand = list(range(ns, nb - nr))
        cand.sort(key=lambda i: (-float(np.float32(scores[g, i])), i))
        out.append(sorted(set(range(ns)) | set(cand[:k]) | set(range(nb - nr, nb))))
    return out


@pytest.mark.parametrize("nb,ns,nr,k", [(40, 1, 2, 5), (40, 0, 0, 7), (12, 2, 3, 7), (9, 1, 1, 9), (64, 3, 4, 1), (30, 1, 1, 0)])
def test_select_brute_force(nb, ns, nr, k):
    scores = _rand(3, nb)
    scores[1, ns + 1:ns + 4] = scores[1, ns + 5]        # some exact ties
    idx, cnt = oracle.select_blocks(scores, ns, nr, k)
    ref = _brute_select(scores, ns, nr, k)
    for g in range(3):
        got = idx[g, :cnt[g]].tolist()
        assert got == ref[g]
        assert (idx[g, cnt[g]:] == -1).all()
        assert got == sorted(got) and len(set(got)) == len(got)
        assert set(range(min(ns, nb))) <= set(got) and set(range(max(nb - nr, 0), nb)) <= set(got)
        assert cnt[g] == min(nb, ns + k + nr)


def test_select_ties_lower_index_and_fp32_rounding():
    # blocks 2..7 are candidates.  4 and 6 tie exactly; 3 and 5 differ only
    # below fp32 resolution (5 is larger in fp64) and must count as a tie.
    s = np.array([[9.0, 9.0, 0.1, 1.0, 2.0, 1.0 + 1e-12, 2.0, 0.2, 9.0]])
    idx, cnt = oracle.select_blocks(s, 2, 1, 1)
    assert idx[0, :cnt[0]].tolist() == [0, 1, 4, 8]          # 4 beats 6: exact tie, lower index
    idx, cnt = oracle.select_blocks(s, 1, 1, 2)
    assert idx[0, :cnt[0]].tolist() == [0, 1, 4, 8]          # with ns = 1, block 1 (9.0) is a candidate
    idx, cnt = oracle.select_blocks(s, 2, 1, 3)
    assert idx[0, :cnt[0]].tolist() == [0, 1, 3, 4, 6, 8]     # 3 beats 5: lower index on fp32 tie


def test_select_planted_blocks_of_tiny_config_appear():
    c = workloads.make_case("tiny_f32", seed=5)
    o = workloads.oracle_views(c, 0)
    kmax, kmin = oracle.block_summarize(o["K"], c["B"])
    sc = oracle.block_scores(o["Q"], kmax, kmin, "mean")
    idx, cnt = oracle.select_blocks(sc, c["ns"], c["nr"], c["k_blocks"])
    assert set(c["planted"][0][0].tolist()) <= set(idx[0, :cnt[0]].tolist())
    assert cnt[0] == 10


# ------------------------------------------------------------------ attention
def _sdpa(q, k, v, mask):
    """torch's scaled_dot_product_attention in fp64 (the routine Section 4.1 names)."""
    q, k, v = (torch.from_numpy(np.ascontiguousarray(x))[None] for x in (q, k, v))
    out = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=torch.from_numpy(mask)[None])
    return out[0].numpy()


def _ancestors(parent, j):
    out = []
    while j >= 0:
        out.append(j)
        j = int(parent[j])
    return out[::-1]


def _small_case(seed, M=9, Hq=4, Hkv=2, D=8, L=48, B=4, tree="uniform"):
    rng = np.random.default_rng(seed)
    Q, K, V = _rand(M, Hq, D, rng=rng), _rand(L, Hkv, D, rng=rng), _rand(L, Hkv, D, rng=rng)
    Kd, Vd = _rand(M, Hkv, D, rng=rng), _rand(M, Hkv, D, rng=rng)
    parent = workloads.make_tree(M, tree, rng)
    return Q, K, V, Kd, Vd, parent


def test_attention_hand_example():
    g = json.load(open(os.path.join(GOLD, "tree_attention_hand_example.json")))
    D = g["D"]
    def key(w):
        return [2 * math.log(w)] + [0.0] * (D - 1)
    def val(x):
        return [float(x), -float(x), 0.0, 1.0]
    K = np.array([[key(w)] for w in g["ctx_w"]])
    Kd = np.array([[key(w)] for w in g["draft_w"]])
    V = np.array([[val(x)] for x in g["v_first_ctx"]])
    Vd = np.array([[val(x)] for x in g["v_first_draft"]])
    Q = np.array([[[c] + g["q_rest"]] for c in g["q_first"]], float)
    parent = np.array(g["parent"], np.int32)
    for name, sel in (("full", None), ("only_block1", (np.array([[1]], np.int32), np.array([1], np.int32)))):
        O, lse, ps = oracle.tree_attention(Q, K, V, Kd, Vd, parent, g["B"], *(sel or (None, None)))
        want = [float(Fraction(x)) for x in g[name]["O_first"]]
        np.testing.assert_allclose(O[:, 0, 0], want, rtol=1e-14)
        np.testing.assert_allclose(O[:, 0, 1], [-w for w in want], rtol=1e-14)
        np.testing.assert_allclose(O[:, 0, 2], 0, atol=1e-15)
        np.testing.assert_allclose(O[:, 0, 3], 1, rtol=1e-14)
        np.testing.assert_allclose(lse[:, 0], np.log(g[name]["sumexp"]), rtol=1e-14)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_attention_select_all_equals_full_attention_sdpa(seed):
    Q, K, V, Kd, Vd, parent = _small_case(seed)
    M, Hq, D = Q.shape
    L, Hkv, _ = K.shape
    G, B = Hq // Hkv, 4
    nb = L // B
    all_idx = np.tile(np.arange(nb, dtype=np.int32), (Hkv, 1))
    O_all, lse_all, _ = oracle.tree_attention(Q, K, V, Kd, Vd, parent, B, all_idx, np.full(Hkv, nb, np.int32))
    O_none, lse_none, _ = oracle.tree_attention(Q, K, V, Kd, Vd, parent, B)
    assert np.array_equal(O_all, O_none) and np.array_equal(lse_all, lse_none)
    # library reference: SDPA over [context ; draft nodes] with an explicit ancestor mask
    mask = np.zeros((M, L + M), bool)
    mask[:, :L] = True
    for j in range(M):
        mask[j, [L + a for a in _ancestors(parent, j)]] = True
    for h in range(Hq):
        g = h // G
        ref = _sdpa(Q[:, h], np.concatenate([K[:, g], Kd[:, g]]), np.concatenate([V[:, g], Vd[:, g]]), mask)
        np.testing.assert_allclose(O_none[:, h], ref, atol=1e-12)


@pytest.mark.parametrize("seed,tree", [(3, "uniform"), (4, "bounded"), (5, "star"), (6, "chain")])
def test_attention_per_path_brute_force(seed, tree):
    """Every root->leaf path, run as ordinary causal attention over
    [kept context ; path tokens], reproduces the rows of the path's nodes."""
    Q, K, V, Kd, Vd, parent = _small_case(seed, tree=tree)
    M, Hq, D = Q.shape
    L, Hkv, _ = K.shape
    G, B = Hq // Hkv, 4
    rng = np.random.default_rng(seed)
    n_sel = 5
    sel = np.stack([np.sort(rng.choice(L // B, n_sel, replace=False)) for _ in range(Hkv)]).astype(np.int32)
    O, lse, ps = oracle.tree_attention(Q, K, V, Kd, Vd, parent, B, sel, np.full(Hkv, n_sel, np.int32))
    np.testing.assert_allclose(ps, 1.0, atol=1e-13)
    leaves = [j for j in range(M) if j not in set(parent.tolist())]
    seen = set()
    for leaf in leaves:
        path = _ancestors(parent, leaf)
        seen |= set(path)
        for h in range(Hq):
            g = h // G
            toks = np.concatenate([np.arange(i * B, (i + 1) * B) for i in sel[g]])
            keys = np.concatenate([K[toks, g], Kd[path, g]])
            vals = np.concatenate([V[toks, g], Vd[path, g]])
            n, p = len(toks), len(path)
            mask = np.ones((p, n + p), bool)
            mask[:, n:] = np.tril(np.ones((p, p), bool))
            ref = _sdpa(Q[path, h], keys, vals, mask)
            np.testing.assert_allclose(O[path, h], ref, atol=1e-12)
            z = (Q[path, h] @ keys.T) / math.sqrt(D)
            z[~mask] = -np.inf
            np.testing.assert_allclose(lse[path, h], torch.logsumexp(torch.from_numpy(z), -1).numpy(), atol=1e-12)
    assert seen == set(range(M))


def test_attention_chain_is_causal_sdpa_and_single_token_decode():
    Q, K, V, Kd, Vd, parent = _small_case(7, M=6, tree="chain")
    M, Hq, D = Q.shape
    L, Hkv, _ = K.shape
    G = Hq // Hkv
    O, _, _ = oracle.tree_attention(Q, K, V, Kd, Vd, parent, 4)
    for h in range(Hq):
        g = h // G
        keys = torch.from_numpy(np.concatenate([K[:, g], Kd[:, g]]))[None]
        vals = torch.from_numpy(np.concatenate([V[:, g], Vd[:, g]]))[None]
        qfull = torch.zeros((1, L + M, D), dtype=torch.float64)
        qfull[0, L:] = torch.from_numpy(Q[:, h])
        ref = torch.nn.functional.scaled_dot_product_attention(qfull, keys, vals, is_causal=True)[0, L:].numpy()
        np.testing.assert_allclose(O[:, h], ref, atol=1e-12)
    # M = 1: plain decode of one token over context + itself
    O1, _, _ = oracle.tree_attention(Q[:1], K, V, Kd[:1], Vd[:1], parent[:1], 4)
    np.testing.assert_allclose(O1, O[:1], atol=1e-14)


def test_attention_invariants():
    Q, K, V, Kd, Vd, parent = _small_case(8, M=10, L=64)
    M, Hq, D = Q.shape
    L, Hkv, _ = K.shape
    B, G = 4, Hq // Hkv
    sel = np.array([[0, 3, 7, 9, 15], [1, 2, 8, 14, 15]], np.int32)
    cnt = np.array([5, 4], np.int32)          # KV head 1 keeps only its first four
    O, lse, ps = oracle.tree_attention(Q, K, V, Kd, Vd, parent, B, sel, cnt)
    np.testing.assert_allclose(ps, 1.0, atol=1e-13)
    # the order of the kept list does not matter
    sel2 = np.array([[9, 0, 15, 7, 3], [8, 2, 1, 14, -1]], np.int32)
    O2, lse2, _ = oracle.tree_attention(Q, K, V, Kd, Vd, parent, B, sel2, cnt)
    np.testing.assert_allclose(O2, O, atol=1e-13)
    # entries past sel_count are ignored (15 for head 1)
    sel3 = sel.copy(); sel3[1, 4] = 5
    assert np.array_equal(oracle.tree_attention(Q, K, V, Kd, Vd, parent, B, sel3, cnt)[0], O)
    # outputs are convex combinations of the attended values
    for h in range(Hq):
        g = h // G
        toks = np.concatenate([np.arange(i * B, (i + 1) * B) for i in sel[g, :cnt[g]]])
        for j in range(M):
            vals = np.concatenate([V[toks, g], Vd[_ancestors(parent, j), g]])
            assert (O[j, h] <= vals.max(0) + 1e-12).all() and (O[j, h] >= vals.min(0) - 1e-12).all()
    # shifting every key by delta adds the constant q.delta to a row's logits: O unchanged,
    # LSE moves by q.delta / sqrt(D)
    delta = _rand(D)
    O4, lse4, _ = oracle.tree_attention(Q, K + delta, V, Kd + delta, Vd, parent, B, sel, cnt)
    np.testing.assert_allclose(O4, O, atol=1e-11)
    np.testing.assert_allclose(lse4 - lse, (Q @ delta) / math.sqrt(D), atol=1e-11)
    # a value that is the same for every key comes back unchanged
    O5, _, _ = oracle.tree_attention(Q, K, np.ones_like(V) * 3.25, Kd, np.ones_like(Vd) * 3.25, parent, B, sel, cnt)
    np.testing.assert_allclose(O5, 3.25, rtol=1e-13)
    # dropping a kept block changes the result (the selection really gates the keys)
    sel6 = sel.copy(); sel6[0, 0] = 1
    assert not np.allclose(oracle.tree_attention(Q, K, V, Kd, Vd, parent, B, sel6, cnt)[0][:, :G], O[:, :G])


def test_attention_star_tree_sees_root_and_self_only():
    Q, K, V, Kd, Vd, parent = _small_case(9, M=5, tree="star")
    O, _, _ = oracle.tree_attention(Q, K, V, Kd, Vd, parent, 4)
    # changing sibling 3's key/value must not change node 2's row, but changes node 3's
    Kd2, Vd2 = Kd.copy(), Vd.copy()
    Kd2[3] += 1.0; Vd2[3] -= 2.0
    O2, _, _ = oracle.tree_attention(Q, K, V, Kd2, Vd2, parent, 4)
    assert np.array_equal(O2[[0, 1, 2, 4]], O[[0, 1, 2, 4]]) and not np.allclose(O2[3], O[3])
    # changing the root changes everyone
    Kd3 = Kd.copy(); Kd3[0] += 1.0
    O3, _, _ = oracle.tree_attention(Q, K, V, Kd3, Vd, parent, 4)
    assert all(not np.allclose(O3[j], O[j]) for j in range(5))


def test_attention_ragged_tail_block():
    # L not a multiple of B: the trailing block holds fewer tokens; nothing past L is read
    Q, K, V, Kd, Vd, parent = _small_case(10, L=46)
    B = 4
    sel = np.array([[0, 11], [5, 11]], np.int32)
    cnt = np.array([2, 2], np.int32)
    O, _, _ = oracle.tree_attention(Q, K, V, Kd, Vd, parent, B, sel, cnt)
    Kp = np.concatenate([K, 1e3 * np.ones((2, 2, 8))]); Vp = np.concatenate([V, 1e3 * np.ones((2, 2, 8))])
    mask_tokens = [list(range(0, 4)) + [44, 45], list(range(20, 24)) + [44, 45]]
    M, Hq, D = Q.shape
    for h in range(Hq):
        g = h // 2
        toks = mask_tokens[g]
        for j in range(M):
            anc = _ancestors(parent, j)
            keys = np.concatenate([K[toks, g], Kd[anc, g]]); vals = np.concatenate([V[toks, g], Vd[anc, g]])
            ref = _sdpa(Q[j:j + 1, h], keys, vals, np.ones((1, len(keys)), bool))
            np.testing.assert_allclose(O[j:j + 1, h], ref, atol=1e-12)


def test_full_verify_refresh_is_the_composition():
    Q, K, V, Kd, Vd, parent = _small_case(11, L=64)
    B = 4
    O, lse, idx, cnt, sc = oracle.full_verify_refresh(Q, K, V, Kd, Vd, parent, B, 1, 2, 4)
    O_ref, lse_ref, _ = oracle.tree_attention(Q, K, V, Kd, Vd, parent, B)
    kmax, kmin = oracle.block_summarize(K, B)
    idx_ref, cnt_ref = oracle.select_blocks(oracle.block_scores(Q, kmax, kmin), 1, 2, 4)
    assert np.array_equal(O, O_ref) and np.array_equal(idx, idx_ref) and np.array_equal(cnt, cnt_ref)
    assert idx.shape == (2, 7) and (cnt == 7).all()


# ---- verification modes and the buffer (Section 3.3, Algorithm 1) ---------------------------

def test_mode_policy_matches_the_hand_worked_example():
    """tests/golden/mode_policy_hand_example.json: the mode sequence written out by hand from
    Section 3.3; also replays the state transitions it implies."""
    g = json.load(open(os.path.join(GOLD, "mode_policy_hand_example.json")))
    names = {"FULL": oracle.MODE_FULL, "PARTIAL": oracle.MODE_PARTIAL, "REFRESH": oracle.MODE_REFRESH}
    budget, margin = g["partial_budget_tokens"], g["pending_margin_tokens"]
    seq_len, ready, pending = g["steps"][0]["seq_len"], False, 0
    for st in g["steps"]:
        assert (seq_len, ready, pending) == (st["seq_len"], st["partial_ready"], st["n_pending"]), st
        mode = oracle.select_mode(seq_len, ready, pending, budget, margin)
        assert mode == names[st["mode"]], (st, mode)
        if mode == oracle.MODE_PARTIAL:
            pending += st["accepted"]
        else:
            pending = 0
            if seq_len > budget:
                ready = True
        seq_len += st["accepted"]


def _ancestor_set(parent, j):
    out = set()
    while j >= 0:
        out.add(j)
        j = parent[j]
    return out


def test_extended_tree_is_a_chain_plus_the_shifted_tree():
    rng = np.random.default_rng(3)
    for n_pending in (0, 1, 7):
        tree = workloads.make_tree(13, "uniform", rng)
        ext = oracle.extend_parents(tree, n_pending)
        assert len(ext) == n_pending + 13 and all(p < i for i, p in enumerate(ext))
        for j in range(13):
            want = set(range(n_pending)) | {a + n_pending for a in _ancestor_set(tree, j)}
            assert _ancestor_set(ext, n_pending + j) == want
        for i in range(n_pending):
            assert _ancestor_set(ext, i) == set(range(i + 1))


def test_pending_tokens_as_chain_prefix_equal_pending_tokens_in_the_cache():
    """The reading behind the buffer (Section 3.2: the four components are handled as one
    continuous KV segment): attending over `cache + pending chain + tree` gives the candidates
    exactly what attending over `cache extended by the pending tokens + tree` gives them."""
    rng = np.random.default_rng(11)
    Hq, Hkv, D, B, L, n_pending, M = 4, 2, 16, 4, 37, 5, 9
    K, V = rng.standard_normal((L, Hkv, D)), rng.standard_normal((L, Hkv, D))
    pk, pv = rng.standard_normal((n_pending, Hkv, D)), rng.standard_normal((n_pending, Hkv, D))
    Q, Kd, Vd = rng.standard_normal((M, Hq, D)), rng.standard_normal((M, Hkv, D)), rng.standard_normal((M, Hkv, D))
    tree = workloads.make_tree(M, "bounded", rng)
    ext = np.array(oracle.extend_parents(tree, n_pending), dtype=np.int32)
    Qe = np.concatenate([rng.standard_normal((n_pending, Hq, D)), Q])   # the pending tokens' queries do not matter
    O1, lse1, _ = oracle.tree_attention(Qe, K, V, np.concatenate([pk, Kd]), np.concatenate([pv, Vd]), ext, B)
    O2, lse2, _ = oracle.tree_attention(Q, np.concatenate([K, pk]), np.concatenate([V, pv]), Kd, Vd,
                                        np.array(tree, dtype=np.int32), B)
    np.testing.assert_allclose(O1[n_pending:], O2, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(lse1[n_pending:], lse2, rtol=1e-11, atol=1e-12)


def test_commit_keeps_exactly_the_accepted_tokens_in_order():
    rng = np.random.default_rng(5)
    Hkv, D, cap, L0, M = 2, 8, 64, 20, 10
    K, V = np.zeros((cap, Hkv, D)), np.zeros((cap, Hkv, D))
    K[:L0], V[:L0] = rng.standard_normal((L0, Hkv, D)), rng.standard_normal((L0, Hkv, D))
    K0, V0 = K.copy(), V.copy()
    L, pk, pv = L0, [], []
    log_k = []          # what the cache must hold behind L0 in the end, written down independently
    pend_log = []
    for step, mode in enumerate([oracle.MODE_PARTIAL, oracle.MODE_PARTIAL, oracle.MODE_REFRESH, oracle.MODE_FULL,
                                 oracle.MODE_PARTIAL]):
        ck, cv = rng.standard_normal((M, Hkv, D)), rng.standard_normal((M, Hkv, D))
        acc = sorted(rng.choice(M, size=int(rng.integers(1, 5)), replace=False).tolist())
        L_before = L
        L, pk, pv = oracle.commit_accepted(K, V, L, pk, pv, ck, cv, acc, mode, cap)
        pend_log += [ck[a] for a in acc]
        if mode == oracle.MODE_PARTIAL:
            assert L == L_before and len(pk) == len(pend_log)
            assert np.array_equal(K, K0) or L_before > L0   # a partial step never writes the cache
        else:
            log_k += pend_log
            pend_log = []
            assert len(pk) == 0 and L == L0 + len(log_k)
    assert np.array_equal(K[:L0], K0[:L0]) and np.array_equal(V[:L0], V0[:L0])
    assert np.array_equal(K[L0:L], np.stack(log_k))
    assert not K[L:].any()                                   # nothing beyond the committed length
    assert len(pk) == len(pend_log) and all(np.array_equal(a, b) for a, b in zip(pk, pend_log))


def test_gathered_cache_gives_the_same_attention_as_the_lists():
    """Section 3.2: the kept tokens form one contiguous KV segment.  Attention over the
    gathered segment (all of it) equals attention over the block lists; the gather itself is
    checked against numpy fancy indexing."""
    rng = np.random.default_rng(21)
    Hq, Hkv, D, B, L, M, n_sel = 4, 2, 8, 4, 46, 7, 5     # 12 blocks, the last one ragged (2 tokens)
    K, V = rng.standard_normal((L, Hkv, D)), rng.standard_normal((L, Hkv, D))
    Q, Kd, Vd = rng.standard_normal((M, Hq, D)), rng.standard_normal((M, Hkv, D)), rng.standard_normal((M, Hkv, D))
    parent = np.array(workloads.make_tree(M, "bounded", rng), dtype=np.int32)
    sel = np.stack([np.array([0, 3, 4, 9, 11]), np.array([1, 2, 7, 10, 11])]).astype(np.int32)
    cnt = np.full(Hkv, n_sel, np.int32)
    Kg, Vg, rows = oracle.gather_blocks(K, V, B, sel, cnt)
    assert rows.tolist() == [4 * B + 2, 4 * B + 2]
    for g in range(Hkv):
        toks = np.concatenate([np.arange(i * B, min((i + 1) * B, L)) for i in sel[g]])
        assert np.array_equal(Kg[:len(toks), g], K[toks, g]) and np.array_equal(Vg[:len(toks), g], V[toks, g])
        assert not Kg[len(toks):, g].any()
    O1, lse1, _ = oracle.tree_attention(Q, K, V, Kd, Vd, parent, B, sel, cnt)
    O2, lse2, _ = oracle.tree_attention(Q, Kg[:rows[0]], Vg[:rows[0]], Kd, Vd, parent, B)
    np.testing.assert_allclose(O1, O2, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse1, lse2, rtol=1e-12, atol=1e-13)


# ------------------------------------------------------------------ finite storage, key-only nodes, list upkeep
def test_commit_with_finite_storage_hand_example():
    g = json.load(open(os.path.join(GOLD, "commit_hand_example.json")))
    for name in ("cache_full", "buffer_full"):
        c = g[name]
        cap = c.get("capacity", 16)
        K, V = np.zeros((cap, 1, 1)), np.zeros((cap, 1, 1))
        K[:c["L"], 0, 0] = np.arange(1, c["L"] + 1)
        V[:] = -K
        pk = [np.full((1, 1), x) for x in c["pending"]]
        pv = [-x for x in pk]
        ck = np.array(c["candidates"]).reshape(-1, 1, 1)
        mode = {"refresh": oracle.MODE_REFRESH, "partial": oracle.MODE_PARTIAL}[c["mode"]]
        L, pk2, pv2 = oracle.commit_accepted(K, V, c["L"], pk, pv, ck, -ck, c["accepted"], mode, cap, c.get("pending_cap"))
        assert L == c["L_after"]
        assert [float(x[0, 0]) for x in pk2] == c["pending_after"] and [float(x[0, 0]) for x in pv2] == [-x for x in c["pending_after"]]
        if "cache_tail_after" in c:
            assert K[c["L"]:L, 0, 0].tolist() == c["cache_tail_after"] and V[c["L"]:L, 0, 0].tolist() == [-x for x in c["cache_tail_after"]]
        assert K[:c["L"], 0, 0].tolist() == list(range(1, c["L"] + 1))
        assert oracle.commit_dropped(c["L"], len(c["pending"]), len(c["accepted"]), mode, cap, c.get("pending_cap")) == c["dropped"]


def test_extend_lists_hand_example():
    g = json.load(open(os.path.join(GOLD, "commit_hand_example.json")))
    for c in g["extend_lists"]:
        src = np.array(c["sel_idx"], np.int32)
        idx, cnt, miss = oracle.extend_lists(src, np.array(c["sel_count"], np.int32), c["L_old"], c["L_new"], c["B"])
        assert idx.tolist() == c["sel_idx_after"] and cnt.tolist() == c["sel_count_after"] and miss.tolist() == c["not_listed"], c["_note"]
        assert src.tolist() == c["sel_idx"]      # the input is not written


def test_key_only_nodes_are_keys_without_query_rows():
    """A node without a query row is attended like any other draft node; its own (absent) output does not
    exist.  Equals the rows of the other nodes when the key-only nodes are given arbitrary queries."""
    rng = np.random.default_rng(17)
    Hq, Hkv, D, B, L, n, M = 4, 2, 8, 4, 23, 3, 6
    K, V = rng.standard_normal((L, Hkv, D)), rng.standard_normal((L, Hkv, D))
    Kd, Vd = rng.standard_normal((n + M, Hkv, D)), rng.standard_normal((n + M, Hkv, D))
    Q = rng.standard_normal((M, Hq, D))
    ext = np.array(oracle.extend_parents(workloads.make_tree(M, "bounded", rng), n), dtype=np.int32)
    sel, cnt = np.array([[0, 2, 5], [1, 3, 5]], np.int32), np.array([3, 3], np.int32)
    O1, lse1, ps1 = oracle.tree_attention(Q, K, V, Kd, Vd, ext, B, sel, cnt, n_key_only=n)
    Qe = np.concatenate([rng.standard_normal((n, Hq, D)), Q])
    O2, lse2, ps2 = oracle.tree_attention(Qe, K, V, Kd, Vd, ext, B, sel, cnt)
    assert O1.shape == (M, Hq, D) and np.array_equal(O1, O2[n:]) and np.array_equal(lse1, lse2[n:])
    np.testing.assert_allclose(ps1, 1.0, rtol=1e-12)


@pytest.mark.parametrize("L_old,m", [(37, 6), (40, 3), (38, 11), (43, 1)])
def test_lists_extended_at_a_commit_keep_every_committed_token(L_old, m):
    """Section 3.3: what a refresh commits stays in the partial cache.  Before the commit the candidates of the
    next step would see `kept blocks + the m tokens as pending chain`; after it they must see the same keys
    through `kept blocks extended by the blocks the m tokens went to` -- no token lost, none gained."""
    rng = np.random.default_rng(100 + L_old)
    Hq, Hkv, D, B, M, cap = 4, 2, 8, 4, 7, 64
    ns, nr, k = 1, 2, 3
    K, V = np.zeros((cap, Hkv, D)), np.zeros((cap, Hkv, D))
    K[:L_old], V[:L_old] = rng.standard_normal((L_old, Hkv, D)), rng.standard_normal((L_old, Hkv, D))
    nb = (L_old + B - 1) // B
    sc = rng.standard_normal((Hkv, nb))
    sel, cnt = oracle.select_blocks(sc, ns, nr, k)                 # what the refresh built for L_old
    sel = np.concatenate([sel, np.full((Hkv, 4), -1, np.int32)], axis=1)   # room for the blocks to come
    pk, pv = rng.standard_normal((m, Hkv, D)), rng.standard_normal((m, Hkv, D))
    Q, Kd, Vd = rng.standard_normal((M, Hq, D)), rng.standard_normal((M, Hkv, D)), rng.standard_normal((M, Hkv, D))
    tree = workloads.make_tree(M, "bounded", rng)
    ext = np.array(oracle.extend_parents(tree, m), dtype=np.int32)
    O1, lse1, _ = oracle.tree_attention(Q, K[:L_old], V[:L_old], np.concatenate([pk, Kd]), np.concatenate([pv, Vd]),
                                        ext, B, sel, cnt, n_key_only=m)
    L_new, _, _ = oracle.commit_accepted(K, V, L_old, list(pk), list(pv), Kd, Vd, [], oracle.MODE_REFRESH, cap)
    assert L_new == L_old + m
    sel2, cnt2, miss = oracle.extend_lists(sel, cnt, L_old, L_new, B)
    assert not miss.any()
    for g in range(Hkv):
        row = sel2[g, :cnt2[g]].tolist()
        assert row == sorted(set(row)) and row[:cnt[g]] == sel[g, :cnt[g]].tolist()
        assert set(range(L_old // B, (L_new - 1) // B + 1)) <= set(row)
    O2, lse2, _ = oracle.tree_attention(Q, K[:L_new], V[:L_new], Kd, Vd, np.array(tree, np.int32), B, sel2, cnt2)
    np.testing.assert_allclose(O1, O2, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(lse1, lse2, rtol=1e-11, atol=1e-12)
    # ... whereas the lists as the refresh left them lose the tokens that opened a new block
    if (L_new - 1) // B > (L_old - 1) // B or L_old % B == 0:
        O3, _, _ = oracle.tree_attention(Q, K[:L_new], V[:L_new], Kd, Vd, np.array(tree, np.int32), B, sel, cnt)
        assert np.abs(O3 - O1).max() > 1e-6
