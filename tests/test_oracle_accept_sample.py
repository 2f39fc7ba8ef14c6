"""Pins of the oracle's stochastic acceptance: the distribution guarantee (the first emitted token
follows softmax(logits / T) exactly), closed-form acceptance probabilities of a single level, the
zero-temperature limit against the (separately pinned) greedy acceptance, numpy's
cumsum/searchsorted for the bonus draw, and hand-checked walks."""
import numpy as np
import pytest

import oracle
import workloads as wl


def _softmax(x):
    e = np.exp(x - x.max())
    return e / e.sum()


def test_first_emitted_token_follows_the_target_distribution():
    """Star tree (all nodes children of the root) over a 7-token vocabulary, 60,000 draws: the
    first token of the step (accepted child's token, else the bonus) must be distributed as p.
    A wrong renormalisation, a missing strike-out or a biased bonus draw shifts these counts by
    far more than the 5-sigma band."""
    V, n_q, N = 7, 3, 60000
    rng = np.random.default_rng(0)
    logits = rng.standard_normal((n_q + 1, V)) * 1.5
    p = _softmax(logits[0] / 0.8)
    draft = np.array([4, 1, 4], dtype=np.int32)          # a duplicated token among the siblings
    parent = np.array([-1, -1, -1], dtype=np.int32)
    lg = np.tile(logits, (N, 1))
    ua, ub = rng.random((N, n_q)), rng.random(N)
    alen, path, bonus, _ = oracle.accept_sample(lg, np.tile(draft, N), parent, N, n_q, 0.8, ua, ub)
    first = np.where(alen > 0, draft[np.maximum(path[:, 0], 0)], bonus)
    counts = np.bincount(first, minlength=V)
    sigma = np.sqrt(N * p * (1 - p))
    assert np.all(np.abs(counts - N * p) <= 5 * sigma), (counts, N * p)
    # closed form of one level: P(accept child 0) = p[4]; P(accept child 1) = p[1] (telescoping);
    # child 2 repeats a struck-out token and can never be accepted
    acc0 = np.mean((alen > 0) & (path[:, 0] == 0))
    acc1 = np.mean((alen > 0) & (path[:, 0] == 1))
    assert abs(acc0 - p[4]) <= 5 * np.sqrt(p[4] * (1 - p[4]) / N)
    assert abs(acc1 - p[1]) <= 5 * np.sqrt(p[1] * (1 - p[1]) / N)
    assert not np.any((alen > 0) & (path[:, 0] == 2))


def test_chain_second_token_follows_its_row():
    """Chain of two: given that node 0 was accepted, the next token (node 1's token or the bonus)
    follows the distribution of row 1."""
    V, N = 5, 40000
    rng = np.random.default_rng(1)
    logits = rng.standard_normal((3, V))
    p1 = _softmax(logits[1])
    draft = np.array([2, 3], dtype=np.int32)
    ua, ub = rng.random((N, 2)), rng.random(N)
    ua[:, 0] = 0.0                                       # u = 0 always accepts a token with p > 0
    alen, path, bonus, _ = oracle.accept_sample(np.tile(logits, (N, 1)), np.tile(draft, N), None, N, 2,
                                                1.0, ua, ub)
    assert np.all(alen >= 1)
    second = np.where(alen == 2, 3, bonus)
    counts = np.bincount(second, minlength=V)
    assert np.all(np.abs(counts - N * p1) <= 5 * np.sqrt(N * p1 * (1 - p1)))


def test_low_temperature_limit_is_greedy_acceptance():
    cfg = wl.Config("as-small", "f32", 4, 1, 16, 3, (((wl.TEXT, 8),),) * 3, 8, 10, True, 32, 50)
    parent = wl.pruned_tree(2, 10, (3, 2, 2))
    rng = np.random.default_rng(2)
    B, n_q, V = 3, 10, 50
    lg = rng.standard_normal((B * (n_q + 1), V))
    ids, _ = oracle.argmax(lg)
    draft = rng.integers(0, V, size=(B, n_q)).astype(np.int32)
    t = ids.reshape(B, n_q + 1)
    for b in range(B):                                   # plant paths of depth 2, 1, 0
        cur = -1
        for _ in range(2 - b):
            kids = np.flatnonzero(parent == cur)
            draft[b, kids[1 % len(kids)]] = t[b, cur + 1]
            cur = kids[1 % len(kids)]
    g_len, g_path, g_bonus = oracle.accept(ids, draft.reshape(-1), parent, B, n_q)
    ua = rng.random((B, n_q)) * 0.98 + 0.01
    s_len, s_path, s_bonus, _ = oracle.accept_sample(lg, draft.reshape(-1), parent, B, n_q, 1e-3, ua,
                                                     rng.random(B) * 0.98 + 0.01)
    np.testing.assert_array_equal(s_len, g_len)
    np.testing.assert_array_equal(s_path, g_path)
    np.testing.assert_array_equal(s_bonus, g_bonus)


def test_bonus_draw_is_inverse_cdf_in_vocabulary_order():
    V = 40
    rng = np.random.default_rng(3)
    lg = rng.standard_normal((1, V)) * 2
    p = _softmax(lg[0])
    for u in (0.0, 1e-9, 0.25, 0.5, 0.999999):
        _, _, bonus, _ = oracle.accept_sample(lg, np.zeros(0, np.int32), None, 1, 0, 1.0,
                                              np.zeros((1, 0)), np.array([u]))
        assert bonus[0] == min(int(np.searchsorted(np.cumsum(p), u, side="left")), V - 1)
    # after a rejection the struck-out token can no longer be drawn and the rest is renormalised
    lg2 = np.vstack([lg, lg])
    x = int(np.argmax(p))
    pr = p.copy(); pr[x] = 0.0
    for u in (0.1, 0.6, 0.95):
        alen, _, bonus, _ = oracle.accept_sample(lg2, np.array([x], np.int32), None, 1, 1, 1.0,
                                                 np.array([[0.999999999]]), np.array([u]))
        assert alen[0] == 0
        assert bonus[0] == int(np.searchsorted(np.cumsum(pr), u * pr.sum(), side="left"))
        assert bonus[0] != x


def test_hand_checked_walk_and_thresholds():
    """V = 4, p = (0.1, 0.2, 0.3, 0.4) on every row (logits = log p).  Root has children 0 (token
    3) and 1 (token 2); node 0 has child 2 (token 0)."""
    p = np.array([0.1, 0.2, 0.3, 0.4])
    lg = np.tile(np.log(p), (4, 1))
    parent = np.array([-1, -1, 0], dtype=np.int32)
    draft = np.array([3, 2, 0], dtype=np.int32)
    run = lambda ua, ub: oracle.accept_sample(lg, draft, parent, 1, 3, 1.0, np.array([ua]), np.array([ub]))  # noqa: E731
    # u0 = 0.39 < 0.4: accept node 0; then child 2: u = 0.11 > 0.1 rejects; bonus from (0,.2,.3,.4)/0.9
    alen, path, bonus, margin = run([0.39, 0.5, 0.11], 0.5)
    assert alen[0] == 1 and path[0].tolist() == [0, -1, -1]
    assert bonus[0] == 2            # 0.5 * 0.9 = 0.45: cdf 0.2, 0.5 -> token 2
    np.testing.assert_allclose(margin[0], 0.01, rtol=1e-9)           # |0.39 - 0.4| / 1 is the tightest
    # u0 = 0.41 rejects token 3 (S = 0.6); node 1: 0.49 * 0.6 = 0.294 <= 0.3 accepts; node 1 is a leaf
    alen, path, bonus, _ = run([0.41, 0.49, 0.0], 0.95)
    assert alen[0] == 1 and path[0].tolist() == [1, -1, -1] and bonus[0] == 3    # 0.95 on the full p
    # both rejected: S = 0.3, bonus from (0.1, 0.2, 0, 0): u = 0.34 -> 0.102 > 0.1 -> token 1
    alen, path, bonus, _ = run([0.41, 0.51, 0.0], 0.34)
    assert alen[0] == 0 and bonus[0] == 1
    alen, path, bonus, _ = run([0.41, 0.51, 0.0], 0.33)
    assert bonus[0] == 0
    with pytest.raises(ValueError):
        oracle.accept_sample(lg, draft, parent, 1, 3, 0.0, np.zeros((1, 3)), np.zeros(1))
