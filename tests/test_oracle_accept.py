"""Pins for the lm_head / argmax / greedy-acceptance oracle (CPU only)."""
import itertools

import numpy as np
import pytest

import workloads as wl


def small_cfg(dtype="f32", hidden=48, vocab=97):
    return wl.Config("S", dtype, 4, 2, 16, 1, None, 8, 4, False, hidden, vocab)


def test_logits_match_numpy_matmul(oracle):
    cfg = small_cfg()
    c = wl.accept_case(cfg, seed=1, batch=3, n_q=4, parent=None)
    lg = oracle.logits(c.hidden, c.lm_head, chunk=10)   # several ragged chunks
    ref = c.hidden.astype(np.float64) @ c.lm_head.astype(np.float64).T
    np.testing.assert_allclose(lg, ref, rtol=0, atol=1e-13)
    ids, margin = oracle.argmax(lg)
    np.testing.assert_array_equal(ids, np.argmax(ref, axis=1))
    srt = np.sort(ref, axis=1)
    np.testing.assert_allclose(margin, srt[:, -1] - srt[:, -2], rtol=0, atol=1e-13)


def test_planted_argmax_by_cauchy_schwarz(oracle):
    """Unit-norm lm_head rows and hidden_r = W[t_r]: <W[v], W[t]> <= 1 with
    equality only at v = t, so the greedy token is t_r."""
    rng = np.random.default_rng(2)
    W = rng.standard_normal((200, 32))
    W /= np.linalg.norm(W, axis=1, keepdims=True)
    t = rng.integers(0, 200, size=9)
    ids, margin = oracle.argmax(oracle.logits(W[t], W))
    np.testing.assert_array_equal(ids, t)
    assert (margin > 0).all()


def test_argmax_ties_lowest_id_and_shift_invariance(oracle):
    rng = np.random.default_rng(3)
    W = rng.standard_normal((50, 16))
    W[37] = W[5]                      # duplicated row: exact tie
    h = 3.0 * W[5][None]
    lg = oracle.logits(h, W)
    ids, margin = oracle.argmax(lg)
    assert ids[0] == 5 and margin[0] == 0.0
    ids2, _ = oracle.argmax(lg + 123.5)   # per-row constant changes nothing
    assert ids2[0] == 5


@pytest.mark.parametrize("k", [1, 2, 3, 6])
def test_chain_all_match_patterns(oracle, k):
    """Brute force: every pattern of per-position match / mismatch.  The
    accepted length is the number of leading matches; the bonus token is the
    target token at the first mismatch (or after the last draft token)."""
    V = 11
    rng = np.random.default_rng(4)
    for pattern in itertools.product([0, 1], repeat=k):
        t = rng.integers(0, V, size=k + 1).astype(np.int32)
        d = np.where(np.array(pattern) == 1, t[:k], (t[:k] + 1) % V).astype(np.int32)
        alen, path, bonus = oracle.accept(t, d, None, 1, k)
        lead = 0
        while lead < k and pattern[lead]:
            lead += 1
        assert alen[0] == lead
        assert list(path[0]) == list(range(lead)) + [-1] * (k - lead)
        assert bonus[0] == t[lead]
        # chain given as a tree: same answer
        a2, p2, b2 = oracle.accept(t, d, wl.chain_parent(k), 1, k)
        assert a2[0] == lead and b2[0] == t[lead] and list(p2[0]) == list(path[0])


def all_parent_arrays(n):
    for combo in itertools.product(*[range(-1, i) for i in range(n)]):
        yield np.array(combo, dtype=np.int32)


def greedy_replay(t, d, parent):
    """Independent statement of losslessness: decode greedily token by token;
    at each step the emitted token is the target's greedy token for the current
    node; continue while some child of the current node drafted that token."""
    n = len(d)
    emitted, cur, path = [], -1, []
    while True:
        tok = int(t[cur + 1])
        emitted.append(tok)
        kids = [j for j in range(n) if int(parent[j]) == cur and int(d[j]) == tok]
        if not kids:
            return emitted, path
        cur = kids[0]
        path.append(cur)


def test_tree_brute_force_small(oracle):
    rng = np.random.default_rng(5)
    V = 3   # tiny vocab so that matches and sibling duplicates are frequent
    for n in range(1, 6):
        for parent in all_parent_arrays(n):
            for _ in range(3):
                t = rng.integers(0, V, size=n + 1).astype(np.int32)
                d = rng.integers(0, V, size=n).astype(np.int32)
                alen, path, bonus = oracle.accept(t, d, parent, 1, n)
                emitted, ref_path = greedy_replay(t, d, parent)
                assert alen[0] == len(ref_path)
                assert list(path[0][:alen[0]]) == ref_path
                assert (path[0][alen[0]:] == -1).all()
                # emitted tokens = drafted tokens along the path + bonus
                assert [int(d[j]) for j in ref_path] + [int(bonus[0])] == emitted


def test_batched_accept_is_per_sequence(oracle):
    rng = np.random.default_rng(6)
    parent = wl.pruned_tree(3, 12, (3, 2, 2))
    n = len(parent)
    B = 5
    t = rng.integers(0, 4, size=B * (n + 1)).astype(np.int32)
    d = rng.integers(0, 4, size=B * n).astype(np.int32)
    alen, path, bonus = oracle.accept(t, d, parent, B, n)
    for b in range(B):
        a1, p1, b1 = oracle.accept(t[b * (n + 1):(b + 1) * (n + 1)], d[b * n:(b + 1) * n],
                                   parent, 1, n)
        assert a1[0] == alen[b] and b1[0] == bonus[b] and list(p1[0]) == list(path[b])


def test_accept_step_planted_prefixes(oracle):
    """End to end on C1's lm_head shape: plant greedy tokens through the hidden
    rows, then draft ids that agree on exactly `a` leading positions."""
    cfg = wl.C1
    c = wl.accept_case(cfg, seed=0, planted=True)
    k = cfg.n_q
    for a in range(k + 1):
        d = c.planted_ids[:k].copy()
        if a < k:
            d[a] = (d[a] + 1) % cfg.vocab
        r = oracle.accept_step(c.hidden, c.lm_head, d, None, 1, k)
        np.testing.assert_array_equal(r["target_ids"], c.planted_ids)
        assert r["margin"].min() > 1e-3
        assert r["accept_len"][0] == a and r["bonus_id"][0] == c.planted_ids[a]
        # tau convention: tokens generated per target call = accepted + 1 bonus
        assert r["accept_len"][0] + 1 == a + 1


def test_one_tree_per_sequence_walks_each_tree(oracle):
    """parent [B, n_q]: the walk of sequence b follows tree b; a greedy replay written here from
    the rule (children of the current node in ascending index, first token match) agrees."""
    rng = np.random.default_rng(11)
    B, V = 4, 6
    trees = np.stack([wl.pruned_tree(20 + i, 10, (3, 2, 2)) for i in range(B)])
    n_q = trees.shape[1]
    for trial in range(50):
        target = rng.integers(0, V, size=B * (n_q + 1)).astype(np.int32)
        draft = rng.integers(0, V, size=B * n_q).astype(np.int32)
        alen, path, bonus = oracle.accept(target, draft, trees, B, n_q)
        for b in range(B):
            t, d, par = target[b * (n_q + 1):(b + 1) * (n_q + 1)], draft[b * n_q:(b + 1) * n_q], trees[b]
            cur, walked = -1, []
            while True:
                kids = [j for j in range(n_q) if par[j] == cur and d[j] == t[cur + 1]]
                if not kids:
                    break
                cur = kids[0]
                walked.append(cur)
            assert alen[b] == len(walked) and list(path[b][:len(walked)]) == walked
            assert bonus[b] == t[cur + 1]
