"""Pins of the oracle's stochastic acceptance against a SAMPLED draft (oracle_accept_sample_q) and
of its counter-based random numbers, against what the mathematics fixes:
  - losslessness: with children drawn i.i.d. from the draft distribution q and fresh uniforms, the
    first emitted token is distributed as the target's p, whatever q is (Monte Carlo);
  - closed forms: q = p accepts always; a single child x is accepted iff u <= p[x] / q[x]; after
    its rejection the bonus token follows max(p - q, 0) normalised (checked against numpy's
    cumulative sum and searchsorted over a grid of uniforms); after two rejections the residual of
    the residual;
  - a chain whose q rows are point masses on the drafted tokens is the deterministic-children rule
    (oracle_accept_sample, pinned on its own);
  - Philox4x32-10 against the published known-answer vectors (tests/golden/)."""
import os

import numpy as np
import pytest

import workloads as wl


def _softmax(x):
    e = np.exp(x - x.max())
    return e / e.sum()


def _dist(rng, V, sharp=1.0):
    return _softmax(rng.standard_normal(V) * sharp)


@pytest.mark.parametrize("m", [1, 2, 3])
def test_first_emitted_token_is_distributed_as_p(oracle, m):
    """m sibling proposals drawn i.i.d. from q at the root."""
    rng = np.random.default_rng(100 + m)
    V, n = 6, 60000
    lg = rng.standard_normal((m + 1, V)) * 1.5
    p = _softmax(lg[0])
    q = _dist(rng, V, 1.2)
    dq = np.tile(q, (m + 1, 1))
    parent = np.full(m, -1, dtype=np.int32)
    counts = np.zeros(V)
    for _ in range(n):
        draft = rng.choice(V, size=m, p=q).astype(np.int32)
        alen, path, bonus, _ = oracle.accept_sample_q(lg, draft, parent, 1, m, 1.0, dq, rng.random((1, m)),
                                                      rng.random(1))
        tok = draft[path[0, 0]] if alen[0] > 0 else bonus[0]
        counts[tok] += 1
    freq = counts / n
    sigma = np.sqrt(p * (1 - p) / n)
    assert np.all(np.abs(freq - p) <= 4.5 * sigma + 1e-4), (freq, p)


def test_chain_emits_the_targets_joint_distribution(oracle):
    """Chain of two sampled draft tokens: the first emitted token follows p0, and given that the
    first draft token x was accepted, the second emitted token follows the target's row of x's
    node: the pair is distributed as sequential sampling from the target."""
    rng = np.random.default_rng(7)
    V, n = 4, 80000
    lg = rng.standard_normal((3, V)) * 1.3
    p0, p1 = _softmax(lg[0]), _softmax(lg[1])
    dq = np.stack([_dist(rng, V), _dist(rng, V), _dist(rng, V)])
    first = np.zeros(V)
    second_given_acc = np.zeros(V)
    n_acc = 0
    for _ in range(n):
        d0 = rng.choice(V, p=dq[0])
        d1 = rng.choice(V, p=dq[1])
        draft = np.array([d0, d1], dtype=np.int32)
        alen, path, bonus, _ = oracle.accept_sample_q(lg, draft, None, 1, 2, 1.0, dq, rng.random((1, 2)), rng.random(1))
        first[d0 if alen[0] >= 1 else bonus[0]] += 1
        if alen[0] >= 1:
            n_acc += 1
            second_given_acc[d1 if alen[0] == 2 else bonus[0]] += 1
    f = first / n
    assert np.all(np.abs(f - p0) <= 4.5 * np.sqrt(p0 * (1 - p0) / n) + 1e-4), (f, p0)
    # row 1 belongs to draft node 0 whatever token it carries, so the second token follows p1
    g = second_given_acc / n_acc
    assert np.all(np.abs(g - p1) <= 4.5 * np.sqrt(p1 * (1 - p1) / n_acc) + 1e-4), (g, p1)


def test_identical_draft_and_target_always_accept(oracle):
    rng = np.random.default_rng(3)
    V, k = 50, 5
    lg = rng.standard_normal((k + 1, V)) * 2
    dq = np.stack([_softmax(r) for r in lg])
    for _ in range(200):
        draft = np.array([rng.choice(V, p=dq[i]) for i in range(k)], dtype=np.int32)
        alen, path, bonus, _ = oracle.accept_sample_q(lg, draft, None, 1, k, 1.0, dq, rng.random((1, k)) * 0.999999,
                                                      rng.random(1))
        assert alen[0] == k and list(path[0]) == list(range(k))


def test_single_child_threshold_and_residuals(oracle):
    rng = np.random.default_rng(5)
    V = 40
    lg = rng.standard_normal((2, V)) * 2
    p = _softmax(lg[0] / 0.8)                       # temperature 0.8
    q = _dist(rng, V, 1.5)
    dq = np.tile(q, (2, 1))
    for x in range(V):
        thr = min(1.0, p[x] / q[x])
        for u in (thr * 0.999, min(thr * 1.001, 0.9999999)):
            alen, _, _, _ = oracle.accept_sample_q(lg, np.array([x], dtype=np.int32), None, 1, 1, 0.8, dq,
                                                   np.array([[u]]), np.array([0.5]))
            assert alen[0] == (1 if u <= p[x] / q[x] else 0), (x, u, thr)
    # bonus after one rejection: inverse CDF of max(p - q, 0), whatever token was rejected
    res = np.maximum(p - q, 0.0)
    cdf = np.cumsum(res)
    x = int(np.argmax(q / p))                      # a token that is rejected for u close to 1
    for ub in np.linspace(0.0005, 0.9995, 400):
        alen, _, bonus, _ = oracle.accept_sample_q(lg, np.array([x], dtype=np.int32), None, 1, 1, 0.8, dq,
                                                   np.array([[0.9999999]]), np.array([ub]))
        assert alen[0] == 0
        assert bonus[0] == int(np.searchsorted(cdf, ub * cdf[-1], side="left"))
    # two siblings rejected: the residual of the residual
    res1 = res / res.sum()
    res2 = np.maximum(res1 - q, 0.0)
    if res2.sum() > 1e-9:
        cdf2 = np.cumsum(res2)
        par = np.array([-1, -1], dtype=np.int32)
        lg3 = np.vstack([lg, lg[:1]])
        dq3 = np.tile(q, (3, 1))
        y = int(np.argmax(q / np.maximum(res1, 1e-300)))
        for ub in np.linspace(0.001, 0.999, 200):
            alen, _, bonus, _ = oracle.accept_sample_q(lg3, np.array([x, y], dtype=np.int32), par, 1, 2, 0.8, dq3,
                                                       np.array([[0.9999999, 0.9999999]]), np.array([ub]))
            assert alen[0] == 0
            assert bonus[0] == int(np.searchsorted(cdf2, ub * cdf2[-1], side="left"))


def test_point_mass_draft_rows_on_a_chain_are_the_deterministic_rule(oracle):
    rng = np.random.default_rng(9)
    V, k, B = 30, 6, 3
    for trial in range(100):
        lg = rng.standard_normal((B * (k + 1), V)) * 2.5
        draft = rng.integers(0, V, size=B * k).astype(np.int32)
        for b in range(B):                         # some drafts on the target's likeliest token
            for j in range(k):
                if rng.random() < 0.6:
                    draft[b * k + j] = int(np.argmax(lg[b * (k + 1) + j]))
        dq = np.zeros_like(lg)
        for b in range(B):
            for j in range(k):
                dq[b * (k + 1) + j, draft[b * k + j]] = 1.0      # row j's only child is node j
        ua, ub = rng.random((B, k)), rng.random(B)
        a = oracle.accept_sample(lg, draft, None, B, k, 1.0, ua, ub)
        c = oracle.accept_sample_q(lg, draft, None, B, k, 1.0, dq, ua, ub)
        for x, y in zip(a[:3], c[:3]):
            np.testing.assert_array_equal(x, y)


def test_one_tree_per_sequence(oracle):
    rng = np.random.default_rng(13)
    V, B = 12, 3
    trees = np.stack([wl.pruned_tree(40 + i, 7, (3, 2)) for i in range(B)])
    n_q = trees.shape[1]
    lg = rng.standard_normal((B * (n_q + 1), V)) * 2
    dq = np.stack([_dist(rng, V) for _ in range(B * (n_q + 1))])
    draft = rng.integers(0, V, size=B * n_q).astype(np.int32)
    ua, ub = rng.random((B, n_q)), rng.random(B)
    own = oracle.accept_sample_q(lg, draft, trees, B, n_q, 1.0, dq, ua, ub)
    for b in range(B):
        one = oracle.accept_sample_q(lg[b * (n_q + 1):(b + 1) * (n_q + 1)], draft[b * n_q:(b + 1) * n_q], trees[b],
                                     1, n_q, 1.0, dq[b * (n_q + 1):(b + 1) * (n_q + 1)], ua[b:b + 1], ub[b:b + 1])
        for x, y in zip(own, one):
            np.testing.assert_array_equal(x[b:b + 1], y)


def test_philox_known_answers_and_uniforms(oracle):
    path = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        np.testing.assert_array_equal(oracle.philox4x32_10(w[:4], w[4:6]), np.array(w[6:], dtype=np.uint32))
    # the uniforms of a call: one block per (sequence, node), first word, top 24 bits
    seed, offset, B, n_q = 0x0123456789ABCDEF, (5 << 32) | 77, 3, 4
    ua, ub = oracle.philox_uniforms(seed, offset, B, n_q)
    key = [seed & 0xFFFFFFFF, seed >> 32]
    for b in range(B):
        for j in range(n_q):
            w = oracle.philox4x32_10([offset & 0xFFFFFFFF, offset >> 32, b, j], key)
            assert ua[b, j] == (int(w[0]) >> 8) / 2.0 ** 24
        w = oracle.philox4x32_10([offset & 0xFFFFFFFF, offset >> 32, b, 0xFFFFFFFF], key)
        assert ub[b] == (int(w[0]) >> 8) / 2.0 ** 24
    assert np.all((ua >= 0) & (ua < 1)) and np.all((ub >= 0) & (ub < 1))
    # different offsets and seeds give different streams; mean of many uniforms ~ 1/2
    big, _ = oracle.philox_uniforms(1, 0, 64, 64)
    assert abs(big.mean() - 0.5) < 0.02 and len(np.unique(big)) > 4000
    other, _ = oracle.philox_uniforms(1, 1, 64, 64)
    assert not np.array_equal(big, other)
