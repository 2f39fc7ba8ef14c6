"""GPU parity of sparrow_accept against the CPU fp64 oracle: target ids, accepted length, path and
bonus token must match bit for bit.

Floating point decides the argmax, so every graded seed must be well conditioned: the oracle's
top-1 minus top-2 margin has to exceed MARGIN on every row (fp32-accumulated bf16 products differ
from fp64 by ~1e-5 on logits of order 1); a seed that is not is reported as such, never silently
accepted.  Exact ties are tested separately with duplicated lm_head rows."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu
MARGIN = 1e-3


@pytest.fixture(scope="module")
def sp():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2602_15318_amd as sp_
    return sp_


from gpu_util import dev, run_accept  # noqa: E402


def _check(res, ref, what):
    assert ref["margin"].min() >= MARGIN, f"{what}: ill-conditioned seed (margin {ref['margin'].min():.2e})"
    for key in ("target_ids", "accept_len", "accept_path", "bonus_id"):
        np.testing.assert_array_equal(res[key], ref[key], err_msg=f"{what}: {key}")


def _planted_drafts(target_ids, parent, B, n_q, accept_lens, vocab, rng):
    """Draft ids that make sequence b accept exactly accept_lens[b] nodes: walk down the tree
    (first child each time), copying the target token into the chosen child and a different token
    into its siblings; everything else random but different from the relevant target."""
    par = wl.chain_parent(n_q) if parent is None else parent
    ids = rng.integers(0, vocab, size=(B, n_q)).astype(np.int32)
    t = target_ids.reshape(B, n_q + 1)
    for b in range(B):
        # first make sure no node matches by accident
        for j in range(n_q):
            while ids[b, j] == t[b, par[j] + 1]:
                ids[b, j] = (ids[b, j] + 1) % vocab
        cur = -1
        for _ in range(accept_lens[b]):
            kids = np.flatnonzero(par == cur)
            if len(kids) == 0:
                break
            pick = kids[len(kids) // 2]
            ids[b, pick] = t[b, cur + 1]
            cur = pick
    return ids.reshape(-1)


def test_c1_fp32_accept(sp, oracle):
    cfg = wl.C1
    c = wl.accept_case(cfg, 0)
    ref = oracle.accept_step(c.hidden, c.lm_head, c.draft_ids, None, 1, cfg.n_q)
    _check(run_accept(sp, c, 1), ref, "C1 random drafts")
    rng = np.random.default_rng(0)
    for a in range(cfg.n_q + 1):
        ids = _planted_drafts(ref["target_ids"], None, 1, cfg.n_q, [a], cfg.vocab, rng)
        r = oracle.accept_step(c.hidden, c.lm_head, ids, None, 1, cfg.n_q)
        assert r["accept_len"][0] == a
        _check(run_accept(sp, c, 1, draft_ids=ids), r, f"C1 planted {a}")


@pytest.mark.parametrize("dtype,H,V,B,n_q,tree", [
    ("f32", 256, 1000, 2, 3, False), ("f32", 64, 37, 1, 0, False),
    ("bf16", 512, 4096, 1, 5, False), ("bf16", 3584, 12345, 1, 8, False),
    ("bf16", 3584, 8192, 8, 6, False), ("bf16", 1024, 20000, 1, 60, True),
    ("bf16", 520, 777, 3, 4, True), ("bf16", 3584, 16, 1, 2, False),
    # 32, 33 and 64 rows: the last single-pass size, and both ends of the paired-workgroup range
    ("bf16", 1024, 9000, 4, 7, False), ("bf16", 1024, 9000, 3, 10, False),
    ("bf16", 3584, 8192, 8, 7, False),
    # hidden 4096: the eight-wavefront k-split instances at 9, 32, 33 and 64 rows (one block of 16
    # rows, one pass of 32, and both ends of the paired-workgroup range)
    ("bf16", 4096, 6000, 1, 8, False), ("bf16", 4096, 6000, 4, 7, False),
    ("bf16", 4096, 6000, 3, 10, False), ("bf16", 4096, 6000, 8, 7, False),
    ("bf16", 4096, 5000, 1, 48, True)])
def test_accept_shapes(sp, oracle, dtype, H, V, B, n_q, tree):
    cfg = wl.Config("A", dtype, 4, 1, 64, B, None, 8, n_q, tree, H, V)
    parent = None
    if tree:
        parent = wl.pruned_tree(7, n_q, (4, 3, 2, 2, 1, 1) if n_q >= 48 else (2, 2))
        n_q = len(parent)
    # first seed of V, V+1000, ... whose oracle margins are all wide enough (decided on the CPU)
    for seed in range(V, V + 5000, 1000):
        c = wl.accept_case(cfg, seed=seed, batch=B, n_q=n_q, parent=parent)
        ref = oracle.accept_step(c.hidden, c.lm_head, c.draft_ids, parent, B, n_q)
        if ref["margin"].min() >= MARGIN:
            break
    W = dev(c.lm_head, dtype)
    _check(run_accept(sp, c, B, lm_head_dev=W), ref, "random drafts")
    if n_q == 0:
        return
    rng = np.random.default_rng(V)
    depth = 1 + max((int(x) for x in _depths(parent, n_q)), default=0)
    for trial in range(3):
        lens = rng.integers(0, depth + 1, size=B)
        ids = _planted_drafts(ref["target_ids"], parent, B, n_q, lens, V, rng)
        r = oracle.accept_step(c.hidden, c.lm_head, ids, parent, B, n_q)
        _check(run_accept(sp, c, B, draft_ids=ids, lm_head_dev=W), r, f"planted {list(lens)}")


def _depths(parent, n_q):
    par = wl.chain_parent(n_q) if parent is None else parent
    d = np.zeros(n_q, dtype=int)
    for i in range(n_q):
        d[i] = 0 if par[i] < 0 else d[par[i]] + 1
    return d


@pytest.mark.parametrize("dtype,H,V,B,nodes", [
    ("bf16", 3584, 8192, 8, 30),      # 8 requests x 30-node trees: 248 logit rows, four 64-row passes
    ("bf16", 4096, 4096, 3, 25),      # 78 rows: one paired pass and one 16-row pass
    ("bf16", 1024, 5000, 5, 12),      # 65 rows on the fallback matrix-core kernel
    ("f32", 256, 1000, 7, 9),         # 70 rows on the plain-ALU kernel
    ("bf16", 3584, 2048, 8, 63),      # 512 rows, the most one call takes
])
def test_accept_one_tree_per_sequence_and_many_rows(sp, oracle, dtype, H, V, B, nodes):
    """Every sequence of the batch has a draft tree of its own (parent [B, n_q]) and the call holds
    more than 64 logit rows: target ids, accepted length, path and bonus token of every sequence
    against the oracle run sequence by sequence, random drafts and planted paths of every depth."""
    branching = (4, 3, 2, 2, 1, 1) if nodes > 12 else (3, 2, 2)
    trees = np.stack([wl.pruned_tree(200 + i, nodes, branching) for i in range(B)])
    n_q = trees.shape[1]
    cfg = wl.Config("A", dtype, 4, 1, 64, B, None, 8, n_q, True, H, V)
    # planted rows (each a scaled lm_head row plus noise): with up to 512 rows, random rows would
    # hardly ever all have a top-1 / top-2 gap above MARGIN
    c = wl.accept_case(cfg, seed=V, batch=B, n_q=n_q, parent=trees, planted=True)
    ref = oracle.accept_step(c.hidden, c.lm_head, c.draft_ids, trees, B, n_q)
    np.testing.assert_array_equal(ref["target_ids"], c.planted_ids)
    W = dev(c.lm_head, dtype)
    _check(run_accept(sp, c, B, lm_head_dev=W), ref, "random drafts")
    rng = np.random.default_rng(V + B)
    t = ref["target_ids"].reshape(B, n_q + 1)
    for trial in range(2):
        ids = rng.integers(0, V, size=(B, n_q)).astype(np.int32)
        want = []
        for b in range(B):
            par = trees[b]
            for j in range(n_q):
                while ids[b, j] == t[b, par[j] + 1]:
                    ids[b, j] = (ids[b, j] + 1) % V
            cur, depth = -1, int(rng.integers(0, 7))
            n_acc = 0
            for _ in range(depth):
                kids = np.flatnonzero(par == cur)
                if len(kids) == 0:
                    break
                pick = kids[int(rng.integers(0, len(kids)))]
                ids[b, pick] = t[b, cur + 1]
                cur = pick
                n_acc += 1
            want.append(n_acc)
        r = oracle.accept_step(c.hidden, c.lm_head, ids.reshape(-1), trees, B, n_q)
        np.testing.assert_array_equal(r["accept_len"], want)
        _check(run_accept(sp, c, B, draft_ids=ids.reshape(-1), lm_head_dev=W), r, f"planted {want}")


@pytest.mark.parametrize("dtype,H", [("f32", 256), ("bf16", 1024), ("bf16", 3584)])
def test_random_trees_over_a_tiny_vocabulary(sp, oracle, dtype, H):
    """Arbitrary tree shapes (every parent drawn uniformly among the earlier nodes and the root,
    one tree per sequence) over a vocabulary of 6 tokens: drafted tokens coincide with target
    tokens all the time, siblings often carry the same token (the lowest node index must win), and
    walks of every depth occur."""
    V, B, n_q = 6, 6, 20
    cfg = wl.Config("A", dtype, 4, 1, 64, B, None, 8, n_q, True, H, V)
    depths = set()
    for seed in range(6):
        rng = np.random.default_rng(700 + seed)
        trees = np.stack([np.array([int(rng.integers(-1, i)) for i in range(n_q)], dtype=np.int32)
                          for _ in range(B)])
        c = wl.accept_case(cfg, seed=seed, batch=B, n_q=n_q, parent=trees, planted=True)
        draft = rng.integers(0, V, size=B * n_q).astype(np.int32)
        ref = oracle.accept_step(c.hidden, c.lm_head, draft, trees, B, n_q)
        _check(run_accept(sp, c, B, draft_ids=draft), ref, f"seed {seed}")
        depths.update(ref["accept_len"].tolist())
        # the same drafts on one shared tree
        ref1 = oracle.accept_step(c.hidden, c.lm_head, draft, trees[0], B, n_q)
        c.parent = trees[0]
        _check(run_accept(sp, c, B, draft_ids=draft), ref1, f"seed {seed}, shared tree")
    assert len(depths) >= 3, depths


def test_exact_ties_take_lowest_id(sp, oracle):
    """Duplicated lm_head rows give bit-equal logits on both sides: the lower id must win, also
    when the duplicates fall into different tiles / wavefronts of the GEMM pass."""
    cfg = wl.Config("A", "bf16", 4, 1, 64, 1, None, 8, 3, False, 512, 9000)
    c = wl.accept_case(cfg, seed=3, planted=True)
    W = c.lm_head.copy()
    pairs = []
    for r, t in enumerate(c.planted_ids):
        other = (int(t) + 4099 + 17 * r) % cfg.vocab
        W[other] = W[t]
        pairs.append((min(int(t), other), max(int(t), other)))
    c.lm_head = W
    ref = oracle.accept_step(c.hidden, W, c.draft_ids, None, 1, 3)
    assert (ref["margin"] == 0).all()
    np.testing.assert_array_equal(ref["target_ids"], [p[0] for p in pairs])
    res = run_accept(sp, c, 1)
    for key in ("target_ids", "accept_len", "accept_path", "bonus_id"):
        np.testing.assert_array_equal(res[key], ref[key])


def test_c5_full_vocab_accept(sp, oracle):
    """The benchmarked lm_head: 152,064 x 3584 bf16, 9 rows, chain of 8; oracle computes the whole
    logit matrix."""
    cfg = wl.C5
    c = wl.accept_case(cfg, 0)
    W = dev(c.lm_head, "bf16")
    ref = oracle.accept_step(c.hidden, c.lm_head, c.draft_ids, None, 1, cfg.n_q)
    _check(run_accept(sp, c, 1, lm_head_dev=W), ref, "C5 random drafts")
    rng = np.random.default_rng(5)
    for a in (0, 3, 8):
        ids = _planted_drafts(ref["target_ids"], None, 1, cfg.n_q, [a], cfg.vocab, rng)
        r = oracle.accept(ref["target_ids"], ids, None, 1, cfg.n_q)
        assert r[0][0] == a
        res = run_accept(sp, c, 1, draft_ids=ids, lm_head_dev=W)
        np.testing.assert_array_equal(res["target_ids"], ref["target_ids"])
        np.testing.assert_array_equal(res["accept_len"], r[0])
        np.testing.assert_array_equal(res["accept_path"], r[1])
        np.testing.assert_array_equal(res["bonus_id"], r[2])


def test_accept_argument_errors(sp):
    import torch
    h = torch.zeros(66, 64, dtype=torch.bfloat16, device="cuda")
    W = torch.zeros(100, 64, dtype=torch.bfloat16, device="cuda")
    ids = torch.zeros(65, dtype=torch.int32, device="cuda")
    with pytest.raises(sp.SparrowError) as e:      # 66 rows > 64
        sp.accept(h, W, ids, None, 1, 65)
    assert e.value.code == -2
    with pytest.raises(sp.SparrowError) as e:      # workspace too small
        sp.accept(h[:4], W, ids[:3], None, 1, 3,
                  workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.code == -3
