"""Pins of the oracle's proposal (softmax + Top-K), pruning and dynamic tree (CPU only)."""
import os

import numpy as np
import pytest
import scipy.special
import torch

from util import O, read_golden


# ------------------------------------------------------------------ softmax + Top-K
def test_softmax_topk_equals_library_sort():
    rng = np.random.default_rng(0)
    for trial in range(20):
        v = rng.standard_normal(977) * 3
        ids, ps = O.softmax_topk(v, 9)
        p = scipy.special.softmax(v)
        want = torch.topk(torch.as_tensor(p), 9)
        assert ids.tolist() == want.indices.tolist()
        np.testing.assert_allclose(ps, want.values.numpy().astype(np.float32), rtol=1e-6)
        assert np.all(np.diff(ps) <= 0) and ps.sum() <= 1.0 + 1e-6


def test_softmax_topk_ties_take_lowest_id():
    v = np.zeros(50)
    v[[7, 3, 40]] = 2.0
    v[[11, 5]] = 1.0
    ids, ps = O.softmax_topk(v, 6)
    assert ids.tolist() == [3, 7, 40, 5, 11, 0]
    assert ps[0] == ps[1] == ps[2] and ps[3] == ps[4]


def test_lemma_cosine_threshold_implies_topk_membership():
    """Sec. 3.2 Lemma / App. A: with ||h_m|| = ||h_v|| = c_h, ||w_r|| <= c_w and
    cos(h_m, h_v) > 1 - (Delta_K / 2c)^2, c = sqrt(2) c_w c_h, the greedy token under h_v
    is inside the Top-K set under h_m.  Checked with the oracle's Top-K."""
    rng = np.random.default_rng(5)
    d, V, K = 24, 300, 6
    hits = 0
    for trial in range(200):
        W = rng.standard_normal((V, d))
        hv = rng.standard_normal(d)
        hv /= np.linalg.norm(hv)
        lv = W @ hv
        order = np.argsort(-lv)
        i_star = order[0]
        delta_k = lv[i_star] - lv[order[K - 1]]
        c = np.sqrt(2.0) * np.max(np.linalg.norm(W, axis=1)) * 1.0
        thr = 1.0 - (delta_k / (2 * c)) ** 2
        # a unit vector at cosine slightly above the threshold
        cosv = min(1.0, thr + (1 - thr) * 0.5 * rng.random())
        u = rng.standard_normal(d)
        u -= (u @ hv) * hv
        u /= np.linalg.norm(u)
        hm = cosv * hv + np.sqrt(max(0.0, 1 - cosv ** 2)) * u
        assert hm @ hv >= thr
        ids, _ = O.softmax_topk(W @ hm, K)
        assert i_star in ids.tolist()
        hits += 1
    assert hits == 200


# ------------------------------------------------------------------ static trees, BC
def _lists(rng, k, kp, vocab=1000):
    ids, ps = [], []
    for _ in range(k):
        t = rng.choice(vocab, size=kp, replace=False)
        p = np.sort(rng.dirichlet(np.ones(kp + 5))[:kp])[::-1]
        ids.append(t.astype(np.int64))
        ps.append(p.astype(np.float32))
    return ids, ps


def test_static_trees_match_block_complexity_table(golden_dir):
    rng = np.random.default_rng(7)
    rows = read_golden(os.path.join(golden_dir, "block_complexity.txt"))
    assert len(rows) == 12
    for row in rows:
        bc, n_nodes, widths = int(row[0]), int(row[1]), [int(x) for x in row[2:]]
        k = len(widths)
        assert O.block_complexity(widths) == bc
        ids, ps = _lists(rng, k, max(widths) + 2)
        params = O.TreeParams(B=n_nodes, k=k, K=max(widths), expand_width=1,
                              static_widths=widths)
        tok, parent, prob = O.build_prune_tree(params, ids, ps, root_tok=-5)
        assert len(tok) == n_nodes
        blk = O.make_block(tok, parent, k, O.LAYOUT_PER_NODE)
        assert blk.n_rows == bc
        # Top-1 expansion: all nodes of depth i hang on the most probable node of depth i-1
        depth = blk.depth[:n_nodes]
        for i in range(1, k + 1):
            level = np.nonzero(depth == i)[0]
            assert len(level) == widths[i - 1]
            prev = np.nonzero(depth == i - 1)[0]
            best_prev = prev[np.argmax(prob[prev])]
            assert set(parent[level].tolist()) == {int(best_prev)}


def test_dynamic_tree_worked_example_counts(golden_dir):
    (row,) = read_golden(os.path.join(golden_dir, "dynamic_tree_example.txt"))
    bc, k, B, top1, top2, kept, ex1, ex2 = [int(x) for x in row]
    assert B == bc // (k + 1) and top1 == B - 1 and top2 == B - 2 and kept == B - 1
    # distributions shaped so that two second-depth trajectories beat the 8th and 9th
    # first-depth tokens: the kept tree is 7 + 2 as in the figure
    p1 = np.array([0.5, 0.1, 0.09, 0.08, 0.07, 0.06, 0.05, 0.01, 0.005, 0.001], np.float32)
    p2 = np.array([0.4, 0.3, 0.01, 0.01, 0.01, 0.01, 0.01, 0.01, 0.005, 0.001], np.float32)
    ids = [np.arange(100, 110), np.arange(200, 210)]
    params = O.TreeParams(B=B, k=k, K=10 ** 6, expand_width=1, prune_parent=False)
    tok, parent, prob = O.build_prune_tree(params, ids, [p1, p2], root_tok=1)
    assert len(tok) == B and len(tok) - 1 == kept
    blk = O.make_block(tok, parent, k, O.LAYOUT_PER_NODE)
    assert blk.n_rows == bc
    d = blk.depth[:B]
    assert (int(np.sum(d == 1)), int(np.sum(d == 2))) == (ex1, ex2)
    assert tok[d == 1].tolist() == list(range(100, 107))
    assert tok[d == 2].tolist() == [200, 201]
    np.testing.assert_array_equal(prob[d == 2], np.float32(0.5) * p2[:2])
    # candidate counts: with no cap, B-1 = 9 tokens are drawn from mask 1 and B-2 = 8 from mask 2
    # (lifting the final selection keeps every candidate, so the draw sizes become visible)
    full_draw = O.TreeParams(B=B, k=k, K=10 ** 6, expand_width=1, prune_parent=False)
    cnt = _candidate_counts(full_draw, ids, [p1, p2])
    assert cnt == [top1, top2]


def _candidate_counts(params, ids, ps):
    """Children drawn per depth, read off a run whose final selection keeps everything:
    same draws (min(K, B-i) per expanded node), final budget lifted."""
    k = params.k
    static = [min(params.K, params.B - i) for i in range(1, k + 1)]
    p = O.TreeParams(B=params.B, k=k, K=params.K, expand_width=params.expand_width,
                     prune_parent=params.prune_parent, static_widths=static)
    tok, parent, _ = O.build_prune_tree(p, ids, ps, root_tok=1)
    d = O.make_block(tok, parent, 0, 0).depth
    return [int(np.sum(d == i)) for i in range(1, k + 1)]


# ------------------------------------------------------------------ pruning
def test_pruner_drops_parent_token_and_pulls_next_best():
    ids = [np.array([9, 4, 5, 6, 7]), np.array([4, 9, 5, 8, 3])]
    ps = [np.array([.4, .3, .1, .05, .01], np.float32), np.array([.5, .2, .1, .05, .01], np.float32)]
    on = O.TreeParams(B=50, k=2, K=3, expand_width=0, prune_parent=True)
    tok, parent, prob = O.build_prune_tree(on, ids, ps, root_tok=9)
    for c in range(1, len(tok)):
        assert tok[c] != tok[parent[c]]
    d = O.make_block(tok, parent, 0, 0).depth
    # depth 1: root token 9 is skipped, the 4th entry is pulled in; still K children
    assert tok[d == 1].tolist() == [4, 5, 6]
    # children of node '4' skip token 4 and take 9, 5, 8; children of '5' skip 5
    kids4 = [int(tok[c]) for c in range(len(tok)) if parent[c] >= 0 and tok[parent[c]] == 4 and d[c] == 2]
    kids5 = [int(tok[c]) for c in range(len(tok)) if parent[c] >= 0 and tok[parent[c]] == 5 and d[c] == 2]
    assert kids4 == [9, 5, 8] and kids5 == [4, 9, 8]
    # probabilities are not renormalised
    assert prob[1] == np.float32(.3)
    off = O.TreeParams(B=50, k=2, K=3, expand_width=0, prune_parent=False)
    tok2, parent2, _ = O.build_prune_tree(off, ids, ps, root_tok=9)
    assert tok2[1:4].tolist() == [9, 4, 5]
    # pruner is a no-op when no repeat is present
    tok3, par3, p3 = O.build_prune_tree(on, [ids[0], np.array([1, 2, 3, 8, 0])], ps, root_tok=77)
    tok4, par4, p4 = O.build_prune_tree(off, [ids[0], np.array([1, 2, 3, 8, 0])], ps, root_tok=77)
    assert tok3.tolist() == tok4.tolist() and par3.tolist() == par4.tolist()
    # optional rule: the last generated token is also dropped below depth 1
    last = O.TreeParams(B=50, k=2, K=3, expand_width=0, prune_parent=True, prune_last=True)
    tok5, par5, _ = O.build_prune_tree(last, ids, ps, root_tok=9)
    d5 = O.make_block(tok5, par5, 0, 0).depth
    assert 9 not in tok5[d5 == 2].tolist()


# ------------------------------------------------------------------ Alg. 1 vs brute force
def _enumerate_all(B, k, K, ids, ps, root_tok, prune, width_one):
    """Independent statement: grow every trajectory (or only the most probable node per
    depth when width_one), score it by the product of float32 probabilities, keep the
    B-1 best trajectories."""
    nodes = [((), np.float32(1.0), root_tok)]          # (path of list positions, P, token)
    level = [nodes[0]]
    everything = []
    for i in range(1, k + 1):
        nxt = []
        parents = level
        if width_one and parents:
            parents = [max(parents, key=lambda n: float(n[1]))]
        for path, P, t_par in parents:
            taken = 0
            for pos, (t, p) in enumerate(zip(ids[i - 1], ps[i - 1])):
                if taken >= min(K, B - i):
                    break
                if prune and int(t) == int(t_par):
                    continue
                nxt.append((path + (int(t),), np.float32(P) * np.float32(p), int(t)))
                taken += 1
        everything += nxt
        level = nxt
    everything.sort(key=lambda n: -float(n[1]))
    return everything[:B - 1]


def _paths_of(tok, parent):
    out = []
    for c in range(1, len(tok)):
        p, x = [], c
        while x > 0:
            p.append(int(tok[x]))
            x = int(parent[x])
        out.append(tuple(p[::-1]))
    return out


@pytest.mark.parametrize("width_one", [True, False])
def test_dynamic_tree_equals_exhaustive_enumeration(width_one):
    rng = np.random.default_rng(11)
    checked = 0
    for trial in range(300):
        k = int(rng.integers(1, 4))
        B = int(rng.integers(2, 9))
        K = int(rng.integers(1, 5))
        prune = bool(rng.integers(0, 2))
        ids, ps = _lists(rng, k, K + 2, vocab=12)       # small vocab: repeats do occur
        root_tok = int(rng.integers(0, 12))
        params = O.TreeParams(B=B, k=k, K=K, expand_width=1 if width_one else 0,
                              prune_parent=prune)
        tok, parent, prob = O.build_prune_tree(params, ids, ps, root_tok)
        want = _enumerate_all(B, k, K, ids, ps, root_tok, prune, width_one)
        got = sorted(zip(_paths_of(tok, parent), [float(x) for x in prob[1:]]))
        assert got == sorted((p, float(P)) for p, P, _ in want)
        # invariants: budget, ancestor closure, (depth, creation) row order
        assert len(tok) <= B and tok[0] == root_tok and parent[0] == -1
        d = O.make_block(tok, parent, 0, 0).depth
        assert np.all(np.diff(d) >= 0)
        for c in range(1, len(tok)):
            assert 0 <= parent[c] < c and prob[c] <= prob[parent[c]]
        checked += 1
    assert checked == 300


def test_single_mask_needs_no_selection():
    """With one mask token the tree is the root plus the B-1 best tokens (Sec. 4.2)."""
    rng = np.random.default_rng(13)
    ids, ps = _lists(rng, 1, 31)
    tok, parent, prob = O.build_prune_tree(O.TreeParams(B=30, k=1, K=10 ** 6), ids, ps, root_tok=-1)
    assert len(tok) == 30 and set(parent[1:].tolist()) == {0}
    assert tok[1:].tolist() == ids[0][:29].tolist()


def test_short_lists_and_depth_limit():
    ids = [np.array([1, 2]), np.array([3])]
    ps = [np.array([.6, .3], np.float32), np.array([.9], np.float32)]
    tok, parent, _ = O.build_prune_tree(O.TreeParams(B=20, k=2, K=5, expand_width=0), ids, ps, 0)
    assert tok.tolist() == [0, 1, 2, 3, 3] and parent.tolist() == [-1, 0, 0, 1, 2]
    tok, parent, _ = O.build_prune_tree(O.TreeParams(B=20, k=2, K=5, expand_width=0), ids, ps, 0,
                                        n_depths=1)
    assert tok.tolist() == [0, 1, 2]
    tok, parent, _ = O.build_prune_tree(O.TreeParams(B=20, k=2, K=5), ids, ps, 0, n_depths=0)
    assert tok.tolist() == [0] and parent.tolist() == [-1]
