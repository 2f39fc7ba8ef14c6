"""The seeded input generators: shapes, layouts and tree validity (CPU only)."""
import numpy as np

import workloads as wl


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, -2.5, 3.1415927],
                 dtype=np.float32)
    r = wl.round_to_bf16(x)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7 -> even mantissa (1.0)
    assert r[2] == 1.0 and r[3] == np.float32(1.0 + 2 ** -6)
    assert (wl.round_to_bf16(r) == r).all()
    assert ((r.view(np.uint32) & 0xFFFF) == 0).all()
    import torch
    t = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(r, t)


def test_fixed_layouts():
    for cfg, L, ntext in ((wl.C1, 512, 64), (wl.C2, 8192, 512), (wl.C3, 26112, 1024),
                          (wl.C5, 26112, 1024)):
        lay = wl.layouts_of(cfg, 0)[0]
        assert wl.layout_length(lay) == L
        ti = wl.text_index(lay)
        assert len(ti) == ntext and (np.diff(ti) > 0).all() and ti[-1] == L - 1


def test_ragged_layouts_follow_recipe():
    lays = wl.ragged_layouts(0)
    assert len(lays) == 8
    for lay in lays:
        L = wl.layout_length(lay)
        assert 4096 <= L <= 16384
        types = wl.position_types(lay)
        vf = (types == wl.VISUAL).mean()
        assert 0.84 <= vf <= 0.98
        runs = [t for t, _ in lay]
        assert all(a != b for a, b in zip(runs[:-1], runs[1:]))
        assert 1 <= sum(1 for t in runs if t == wl.TEXT) <= 4
        assert types[-1] == wl.TEXT
    assert wl.ragged_layouts(0) == lays and wl.ragged_layouts(1) != lays


def test_pruned_tree_is_valid_and_deep():
    p = wl.pruned_tree(0)
    assert len(p) == 60 and (p < np.arange(60)).all() and (p >= -1).all()
    depth = np.zeros(60, dtype=int)
    for i in range(60):
        depth[i] = 1 if p[i] < 0 else depth[p[i]] + 1
    assert depth.max() == 6
    assert (np.diff(depth) >= 0).all()         # level order
    # branching never exceeds the per-level budget 4,3,2,2,1,1
    budget = [4, 3, 2, 2, 1, 1]
    for i in range(-1, 60):
        kids = np.flatnonzero(p == i)
        lvl = 0 if i < 0 else depth[i]
        assert len(kids) <= (budget[lvl] if lvl < 6 else 0)


def test_cases_are_seeded_and_storage_exact():
    a = wl.verify_case(wl.C2, seed=0)
    b = wl.verify_case(wl.C2, seed=0)
    c = wl.verify_case(wl.C2, seed=1)
    np.testing.assert_array_equal(a.k, b.k)
    assert not np.array_equal(a.k, c.k)
    assert a.k.shape == (8197, 4, 128) and a.q.shape == (5, 28, 128)
    assert ((a.k.view(np.uint32) & 0xFFFF) == 0).all()
    d = wl.draft_case(wl.C4, seed=0)
    assert d.q.shape == (8, 28, 128) and d.cu_text[-1] == len(d.text_idx)
    for b_ in range(8):
        ti = d.text_idx[d.cu_text[b_]:d.cu_text[b_ + 1]]
        assert ti[-1] == d.cu_seqlens[b_ + 1] - d.cu_seqlens[b_] - 1
    w1 = wl.lm_head_weights(wl.C1)
    assert w1.shape == (1024, 256) and abs(float(w1.std()) - 0.02) < 1e-3


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a one-GPU program: --gpus N with N > 1 exits with a message (no GPU needed to
    find that out)."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode == 2
    assert "one GPU" in res.stderr and res.stdout.strip() == ""
