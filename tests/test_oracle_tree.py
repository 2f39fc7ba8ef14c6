"""Pins of the oracle's dynamic draft-tree construction: library top-k / log-softmax, a brute
force over all token sequences of a small Markov "draft model" (without pruning, the kept nodes
are exactly the most probable prefixes), structural invariants, hand-checked small cases."""
import itertools

import numpy as np
import torch
from scipy.special import log_softmax

import oracle


def test_topk_logprob_against_torch_and_scipy():
    rng = np.random.default_rng(0)
    lg = rng.standard_normal((5, 300)) * 2
    ids, logp, margin = oracle.topk_logprob(lg, 7)
    tv, ti = torch.topk(torch.from_numpy(lg), 7, dim=1)
    np.testing.assert_array_equal(ids, ti.numpy())
    ls = log_softmax(lg, axis=1)
    np.testing.assert_allclose(logp, np.take_along_axis(ls, ids.astype(np.int64), axis=1), rtol=1e-12, atol=1e-12)
    srt = -np.sort(-lg, axis=1)[:, :8]
    np.testing.assert_allclose(margin, (srt[:, :-1] - srt[:, 1:]).min(axis=1), rtol=1e-12)
    # ties: equal logits come out in increasing token id, and the margin says so
    lg2 = np.zeros((1, 10)); lg2[0, [7, 2, 5]] = 3.0; lg2[0, 9] = 1.0
    ids, logp, margin = oracle.topk_logprob(lg2, 4)
    assert ids[0].tolist() == [2, 5, 7, 9] and margin[0] == 0.0
    np.testing.assert_allclose(np.exp(logp[0]).sum() + 6 * np.exp(-np.log(3 * np.e ** 3 + np.e + 6)), 1.0, rtol=1e-12)


def _markov(V, rng):
    P = rng.random((V + 1, V)) ** 3 + 1e-3          # row V: distribution after the root
    return np.log(P / P.sum(axis=1, keepdims=True))


def _grow(logP, width, depth, total):
    """Drive the oracle's pool with a Markov draft: candidates of a node = top `width` next tokens."""
    V = logP.shape[1]
    pool = oracle.TreePool(width, depth)
    ids, lp, _ = oracle.topk_logprob(logP[V:V + 1], width)
    front = pool.expand(ids, lp)
    for _ in range(depth - 1):
        rows = logP[pool.tok[front]]
        ids, lp, _ = oracle.topk_logprob(rows, width)
        front = pool.expand(ids, lp)
    return pool, pool.select(total)


def test_without_pruning_the_kept_nodes_are_the_most_probable_prefixes():
    """width = V: every child of every frontier node is a candidate, but the frontier itself is
    still cut to `width` nodes per level; with V = 4 and depth 3 choose the Markov table so that the
    brute-force top prefixes all descend from frontier nodes (checked), then the kept set must be
    the `total` most probable prefixes of length <= depth over all 4 + 16 + 64 sequences."""
    V, depth, total = 4, 3, 12
    rng = np.random.default_rng(3)
    logP = _markov(V, rng)
    pool, (parent, ids, pidx) = _grow(logP, V, depth, total)
    # brute force: log-probability of every prefix
    allp = {}
    for L in range(1, depth + 1):
        for seq in itertools.product(range(V), repeat=L):
            s, prev = 0.0, V
            for t in seq:
                s += logP[prev, t]; prev = t
            allp[seq] = s
    best = sorted(allp.items(), key=lambda kv: -kv[1])[:total]
    # prefixes of the kept nodes, from parent[] and ids
    kept = []
    for i in range(len(ids)):
        seq, j = [], i
        while j >= 0:
            seq.append(int(ids[j])); j = parent[j]
        kept.append(tuple(reversed(seq)))
    got = sorted(((k, allp[k]) for k in kept), key=lambda kv: -kv[1])
    # the frontier cut can only lose prefixes whose parent was not among the `width` best of its
    # level; make sure this table does not hit that case, then compare
    lvl2 = sorted(((k, v) for k, v in allp.items() if len(k) == 2), key=lambda kv: -kv[1])[:V]
    assert all(k[:2] in dict(lvl2) for k, _ in best if len(k) == 3), "pick another seed"
    assert [k for k, _ in got] == [k for k, _ in best]
    np.testing.assert_allclose([v for _, v in got], [v for _, v in best], rtol=1e-12)
    np.testing.assert_allclose(pool.score[pidx], [allp[k] for k in kept], rtol=1e-12)


def test_structure_of_the_paper_configurations():
    """total-depth-width = 30-4-8, 48-5-10, 25-5-8 on a 50-token Markov draft."""
    rng = np.random.default_rng(4)
    logP = _markov(50, rng)
    for total, depth, width in ((30, 4, 8), (48, 5, 10), (25, 5, 8)):
        pool, (parent, ids, pidx) = _grow(logP, width, depth, total)
        assert pool.n == width + (depth - 1) * width * width
        assert len(parent) == total and np.all(parent < np.arange(total)) and np.all(parent >= -1)
        assert np.all(np.diff(pidx) > 0)                               # pool order kept
        sc = pool.score[pidx]
        assert np.all(sc[parent[parent >= 0]] >= sc[parent >= 0])      # a child never beats its parent
        left_out = np.setdiff1d(np.arange(pool.n), pidx)
        assert pool.score[left_out].max() <= sc.min()                  # the best `total` nodes
        dep = np.zeros(total, dtype=int)
        for i in range(total):
            dep[i] = 1 if parent[i] < 0 else dep[parent[i]] + 1
        assert dep.max() <= depth and np.sum(dep == 1) <= width
        # siblings carry distinct tokens
        for p in set(parent.tolist()):
            kids = ids[parent == p]
            assert len(set(kids.tolist())) == len(kids)
        # frontier of every level: `width` distinct pool entries of that level
        assert len(set(pool.front.tolist())) == width


def test_hand_checked_expand_and_select():
    pool = oracle.TreePool(2, 2)
    f0 = pool.expand(np.array([[7, 3]]), np.log(np.array([[0.6, 0.3]])))
    assert f0.tolist() == [0, 1] and pool.par[:2].tolist() == [-1, -1]
    f1 = pool.expand(np.array([[1, 2], [4, 5]]), np.log(np.array([[0.5, 0.4], [0.9, 0.05]])))
    # scores: 0.30, 0.24 (children of node 0), 0.27, 0.015 (children of node 1)
    np.testing.assert_allclose(np.exp(pool.score[:6]), [0.6, 0.3, 0.30, 0.24, 0.27, 0.015], rtol=1e-12)
    assert f1.tolist() == [2, 4] and pool.par[2:6].tolist() == [0, 0, 1, 1]
    parent, ids, pidx = pool.select(4)
    # best four: 0.6, 0.3 (pool 1), 0.30 (pool 2) -- tie in value? no: 0.3 vs 0.30 are log(0.3) and
    # log(0.6)+log(0.5): equal up to rounding, so do not rely on their order; the fourth is 0.27
    assert sorted(pidx.tolist()) == [0, 1, 2, 4]
    assert parent.tolist() == [-1, -1, 0, 1] and ids.tolist() == [7, 3, 1, 4]
    parent, ids, pidx = pool.select(100)
    assert len(parent) == 6 and parent.tolist() == [-1, -1, 0, 0, 1, 1]
