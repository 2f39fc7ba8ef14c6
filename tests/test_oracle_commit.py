"""Pins of the oracle's post-accept commit: numpy fancy indexing on a labelled cache, the chain
case (an accepted chain prefix is already in place), overlapping moves, untouched rows."""
import numpy as np

import oracle
import workloads as wl


def _labelled(T, row):
    """cache[t, x] = 1000 t + x: every element names its original place."""
    return (1000.0 * np.arange(T)[:, None] + np.arange(row)[None, :]).astype(np.float64)


def test_commit_moves_path_rows_behind_the_context():
    n_q = 6
    cu = np.array([0, 10 + n_q, 10 + n_q + 3 + n_q, 10 + n_q + 3 + n_q + 0 + n_q], dtype=np.int32)
    path = np.array([[1, 2, 5, -1, -1, -1], [3, -1, -1, -1, -1, -1], [0, 1, 2, 3, 4, 5]], dtype=np.int32)
    alen = np.array([3, 1, 6], dtype=np.int32)
    c = _labelled(int(cu[-1]), 8)
    out = oracle.kv_commit(c, cu, n_q, path, alen)
    ref = c.copy()
    for b in range(3):
        first = cu[b + 1] - n_q
        ref[first + np.arange(alen[b])] = c[first + path[b, :alen[b]]]      # library gather/scatter
    np.testing.assert_array_equal(out, ref)
    # sequence 0: rows 10, 11, 12 now hold former rows 11, 12, 15 -- 11 and 12 are both a source
    # and a destination (an in-place, in-order copy that read row 11 after writing it would fail)
    assert out[10, 0] == 11000 and out[11, 0] == 12000 and out[12, 0] == 15000
    assert out[13, 0] == 13000                                              # not accepted: as before
    np.testing.assert_array_equal(out[:10], c[:10])                         # context untouched


def test_commit_of_a_chain_prefix_is_the_identity():
    n_q = 5
    cu = np.array([0, 7 + n_q], dtype=np.int32)
    c = _labelled(12, 4)
    for k in range(n_q + 1):
        path = np.full((1, n_q), -1, dtype=np.int32)
        path[0, :k] = np.arange(k)
        np.testing.assert_array_equal(oracle.kv_commit(c, cu, n_q, path, np.array([k])), c)


def test_commit_on_tree_paths_from_the_accept_oracle():
    """Paths produced by the acceptance oracle itself on a planted tree case."""
    cfg = wl.Config("commit", "f32", 4, 1, 16, 2, (((wl.TEXT, 20),), ((wl.TEXT, 9),)), 8, 12, True, 32, 64)
    parent = wl.pruned_tree(3, 12, (3, 2, 2))
    rng = np.random.default_rng(0)
    target = rng.integers(0, 64, size=(2, 13)).astype(np.int32)
    draft = rng.integers(0, 64, size=(2, 12)).astype(np.int32)
    for b in range(2):                       # plant a path of depth 3 / 2
        cur = -1
        for _ in range(3 - b):
            kids = np.flatnonzero(parent == cur)
            draft[b, kids[-1]] = target[b, cur + 1]
            cur = kids[-1]
    alen, path, _ = oracle.accept(target.reshape(-1), draft.reshape(-1), parent, 2, 12)
    assert alen.tolist() == [3, 2]
    cu = np.array([0, 20 + 12, 20 + 12 + 9 + 12], dtype=np.int32)
    c = _labelled(int(cu[-1]), 16)
    out = oracle.kv_commit(c, cu, 12, path, alen)
    for b in range(2):
        first = cu[b + 1] - 12
        for j in range(alen[b]):
            assert out[first + j, 0] == 1000.0 * (first + path.reshape(2, 12)[b, j])
    hid = _labelled(2 * 13, 32)
    nh = oracle.next_hidden(hid, 2, 12, path, alen)
    p2 = path.reshape(2, 12)
    assert nh[0, 0] == 1000.0 * (1 + p2[0, 2]) and nh[1, 0] == 1000.0 * (13 + 1 + p2[1, 1])
    nh0 = oracle.next_hidden(hid, 2, 12, path, np.array([0, 0]))
    assert nh0[0, 0] == 0.0 and nh0[1, 0] == 13000.0          # nothing accepted: row 0 of the sequence
