"""GPU parity of sparrow_accept_sample (temperature > 0) against the CPU fp64 oracle.

Floating point decides integers here (accept / reject, the bonus token), so every graded case
must be well conditioned: the oracle reports the smallest distance of any decision from its
threshold, relative to the remaining probability mass, and a case is graded bit for bit only if
that margin is at least MARGIN -- the device's logits (fp32-accumulated bf16 products) and its
fp32 exponentials differ from the oracle's by ~1e-5 relative.  A seed that is not well conditioned
is replaced by the next one, decided on the CPU; none qualifying fails the test.  A flat
full-vocabulary row (every token ~1e-5: no draw can be well conditioned) is checked for validity
instead: the device's bonus token must own the target of the inverse CDF within a tolerance."""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu
MARGIN = 1e-4


@pytest.fixture(scope="module")
def sp():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2602_15318_amd as sp_
    return sp_


from gpu_util import dev  # noqa: E402


def _case(cfg, seed, B, n_q, parent, vocab, temperature, plant):
    """Hidden rows, lm_head, drafts and uniforms.  `plant`: fraction of nodes whose drafted token
    is the row's most likely token (so that walks of every depth occur)."""
    ac = wl.accept_case(cfg, seed, vocab=vocab, batch=B, n_q=n_q, parent=parent, planted=plant > 0)
    rng = np.random.default_rng(seed + 77)
    draft = ac.draft_ids.reshape(B, n_q).copy()
    par = wl.chain_parent(n_q) if parent is None else parent
    if plant > 0:
        t = ac.planted_ids.reshape(B, n_q + 1)
        for b in range(B):
            for j in range(n_q):
                if rng.random() < plant:
                    draft[b, j] = t[b, par[j] + 1]
    ua = rng.random((B, n_q)).astype(np.float32)
    ub = rng.random(B).astype(np.float32)
    return ac, draft.reshape(-1).astype(np.int32), ua, ub


def _damped(hidden, H, V, dtype):
    """Planted rows are 50 x an lm_head row (|row|^2 ~ 0.0004 H): the planted logit, 0.02 H, dwarfs
    the rest and nothing is ever rejected.  Rescale so that it sits about 1 above log V, where the
    planted token holds roughly half of the mass and walks accept and reject.  The result is
    rounded to the storage type, so both sides still read the same bits."""
    f = (np.log(V) + 1.0) / (0.02 * H)
    return wl.to_storage(hidden * np.float32(f), dtype)


def _run(sp, ac, draft, ua, ub, parent, B, n_q, temperature):
    dt = ac.cfg.dtype
    r = sp.accept_sample(dev(ac.hidden, dt), dev(ac.lm_head, dt), dev(draft),
                         None if parent is None else dev(parent), B, n_q, temperature,
                         dev(ua), dev(ub))
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in r.items()}


CASES = [
    # dtype, H, V, B, n_q, tree, T, plant
    ("f32", 256, 200, 2, 4, False, 1.0, 0.0),
    ("f32", 256, 1000, 3, 6, False, 0.7, 0.6),
    ("f32", 256, 1024, 1, 12, True, 1.0, 0.5),
    ("bf16", 512, 777, 2, 8, False, 1.0, 0.5),
    ("bf16", 512, 4096, 2, 12, True, 0.5, 0.7),
    ("bf16", 3584, 4096, 1, 8, False, 1.0, 0.6),       # k-split lm_head
    ("bf16", 3584, 2048, 2, 20, True, 1.0, 0.6),       # 42 rows: two passes of the k-split kernel
    ("bf16", 1024, 3000, 1, 8, False, 2.0, 0.5),       # fallback matrix-core lm_head
    ("bf16", 4096, 4096, 1, 8, False, 1.0, 0.6),       # k-split lm_head, eight wavefronts
    ("bf16", 4096, 2048, 2, 20, True, 1.0, 0.6),       # 42 rows: its paired-workgroup pass
]


@pytest.mark.parametrize("dtype,H,V,B,n_q,tree,T,plant", CASES)
def test_accept_sample_matches_oracle(sp, oracle, dtype, H, V, B, n_q, tree, T, plant):
    cfg = wl.Config("as", dtype, 4, 1, 64, B, (((wl.TEXT, 8),),) * B, 8, n_q, tree, H, V)
    parent = wl.pruned_tree(9, n_q, (3, 2, 2, 1, 1, 1)) if tree else None
    if tree:
        assert len(parent) == n_q
    graded = 0
    for seed in range(8):
        ac, draft, ua, ub = _case(cfg, seed, B, n_q, parent, V, T, plant)
        hidden = _damped(ac.hidden, H, V, dtype)
        ac.hidden = hidden
        ref = oracle.accept_sample_step(hidden, ac.lm_head, draft, parent, B, n_q, T, ua, ub)
        if ref["margin"].min() < MARGIN:
            continue
        res = _run(sp, ac, draft, ua, ub, parent, B, n_q, T)
        for key in ("accept_len", "accept_path", "bonus_id"):
            np.testing.assert_array_equal(res[key], ref[key], err_msg=f"seed {seed}: {key}")
        graded += 1
        if graded == 3:
            break
    assert graded >= 2, "fewer than two well-conditioned seeds among 8"


def test_accept_sample_one_tree_per_sequence(sp, oracle):
    """parent [B, n_q]: every sequence walks its own tree (70 logit rows: two passes of lm_head)."""
    dtype, H, V, B, nodes, T = "bf16", 3584, 2048, 5, 13, 1.0
    trees = np.stack([wl.pruned_tree(300 + i, nodes, (3, 2, 2, 1, 1, 1)) for i in range(B)])
    n_q = trees.shape[1]
    cfg = wl.Config("as", dtype, 4, 1, 64, B, (((wl.TEXT, 8),),) * B, 8, n_q, True, H, V)
    graded = 0
    for seed in range(12):
        # drafts planted along each sequence's own tree
        ac = wl.accept_case(cfg, seed, vocab=V, batch=B, n_q=n_q, parent=trees, planted=True)
        rng = np.random.default_rng(seed + 77)
        draft = ac.draft_ids.reshape(B, n_q).copy()
        t = ac.planted_ids.reshape(B, n_q + 1)
        for b in range(B):
            for j in range(n_q):
                if rng.random() < 0.6:
                    draft[b, j] = t[b, trees[b, j] + 1]
        draft = draft.reshape(-1).astype(np.int32)
        ua = rng.random((B, n_q)).astype(np.float32)
        ub = rng.random(B).astype(np.float32)
        hidden = _damped(ac.hidden, H, V, dtype)
        ref = oracle.accept_sample_step(hidden, ac.lm_head, draft, trees, B, n_q, T, ua, ub)
        if ref["margin"].min() < MARGIN:
            continue
        r = sp.accept_sample(dev(hidden, dtype), dev(ac.lm_head, dtype), dev(draft), dev(trees), B, n_q, T,
                             dev(ua), dev(ub))
        torch.cuda.synchronize()
        for key in ("accept_len", "accept_path", "bonus_id"):
            np.testing.assert_array_equal(r[key].cpu().numpy(), ref[key], err_msg=f"seed {seed}: {key}")
        graded += 1
        if graded == 2:
            break
    assert graded >= 1, "no well-conditioned seed among 12"


def test_accept_sample_walk_depths_are_exercised(oracle):
    """The cases above are only worth something if walks of different depths, rejections followed
    by acceptances, and bonus draws after strike-outs all occur: count them on the CPU (the test
    needs no GPU; it sits here because it vouches for the cases of this file)."""
    depths, after_reject = set(), 0
    for dtype, H, V, B, n_q, tree, T, plant in CASES[:5]:
        cfg = wl.Config("as", dtype, 4, 1, 64, B, (((wl.TEXT, 8),),) * B, 8, n_q, tree, H, V)
        parent = wl.pruned_tree(9, n_q, (3, 2, 2, 1, 1, 1)) if tree else None
        for seed in range(8):
            ac, draft, ua, ub = _case(cfg, seed, B, n_q, parent, V, T, plant)
            hidden = _damped(ac.hidden, H, V, dtype)
            ref = oracle.accept_sample_step(hidden, ac.lm_head, draft, parent, B, n_q, T, ua, ub)
            depths.update(ref["accept_len"].tolist())
            par = wl.chain_parent(n_q) if parent is None else parent
            for b in range(B):
                p = ref["accept_path"].reshape(B, n_q)[b]
                for j in range(ref["accept_len"][b]):
                    sibs = np.flatnonzero(par == par[p[j]])
                    after_reject += int(p[j] != sibs[0])
    assert {0, 1, 2, 3} <= depths and after_reject >= 3, (depths, after_reject)


def test_full_vocabulary_peaked_and_flat(sp, oracle):
    """C5's lm_head (152,064 x 3584), chain of 8.  Peaked rows (planted): graded bit for bit.
    Flat rows (random hidden): the bonus token must be a valid inverse-CDF draw within 1e-5 of
    the row's mass."""
    cfg = wl.C5
    n_q, V = cfg.n_q, cfg.vocab
    W = wl.lm_head_weights(cfg, 0)
    ac, draft, ua, ub = _case(cfg, 0, 1, n_q, None, V, 1.0, 0.5)
    ac.lm_head = W
    ac.hidden = _damped(ac.hidden, cfg.hidden, V, "bf16")
    Wd = dev(W, "bf16")
    lg = oracle.logits(ac.hidden, W)
    alen, path, bonus, margin = oracle.accept_sample(lg, draft, None, 1, n_q, 1.0, ua, ub)
    assert margin.min() >= 1e-5, f"ill-conditioned ({margin.min():.2e}): pick another seed"
    r = sp.accept_sample(dev(ac.hidden, "bf16"), Wd, dev(draft), None, 1, n_q, 1.0, dev(ua), dev(ub))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(r["accept_len"].cpu().numpy(), alen)
    np.testing.assert_array_equal(r["accept_path"].cpu().numpy(), path)
    np.testing.assert_array_equal(r["bonus_id"].cpu().numpy(), bonus)
    # flat: random hidden rows, random drafts (all rejected with overwhelming probability)
    rng = np.random.default_rng(5)
    hidden = wl.to_storage(rng.standard_normal((n_q + 1, cfg.hidden), dtype=np.float32), "bf16")
    draft = rng.integers(0, V, size=n_q).astype(np.int32)
    for u in (0.0, 0.123456, 0.5, 0.999):
        ua = np.full((1, n_q), 0.9, dtype=np.float32)
        ub = np.array([u], dtype=np.float32)
        r = sp.accept_sample(dev(hidden, "bf16"), Wd, dev(draft), None, 1, n_q, 1.0, dev(ua), dev(ub))
        torch.cuda.synchronize()
        lg = oracle.logits(hidden[:1], W)[0]
        p = np.exp(lg - lg.max()); p /= p.sum()
        assert r["accept_len"].item() == 0 and p[draft[0]] < 0.5
        p[draft[0]] = 0.0                                   # struck out by the rejection
        S = p.sum()
        cdf = np.cumsum(p)
        t = int(r["bonus_id"].item())
        target = float(ub[0]) * S
        lo = cdf[t - 1] if t > 0 else 0.0
        assert p[t] > 0 and lo - 1e-5 * S <= target <= cdf[t] + 1e-5 * S, (u, t, lo, target, cdf[t])


def test_accept_sample_argument_errors(sp):
    h = torch.zeros(3, 256, device="cuda")
    W = torch.zeros(100, 256, device="cuda")
    d = torch.zeros(2, dtype=torch.int32, device="cuda")
    ua, ub = torch.zeros(1, 2, device="cuda"), torch.zeros(1, device="cuda")
    with pytest.raises(sp.SparrowError) as e:
        sp.accept_sample(h, W, d, None, 1, 2, 0.0, ua, ub)
    assert e.value.code == -1 and "temperature" in str(e.value)
    with pytest.raises(sp.SparrowError) as e:
        sp.accept_sample(h, W, d, None, 1, 2, 1.0, ua, ub, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.code == -3
