"""GPU parity of the two attention entry points against the CPU fp64 oracle, element by element
on the same seeded inputs, through the C-ABI."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sp():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2602_15318_amd as sp_
    return sp_


from gpu_util import check_attn, dev, host, run_draft, run_verify  # noqa: E402

# lse is an fp32 output.  Matrix-core path: the row sums add probabilities rounded to bf16 (2^-9
# relative each, so at most ln(1 + 2^-9) = 2e-3 on lse if every rounding went the same way) on top
# of fp32 rounding of the scores (~1e-4 at |score| ~ 30).
LSE_TOL = {"f32": 2e-5, "bf16": 4e-3}


def _verify_and_check(sp, oracle, c, what):
    out, lse = run_verify(sp, c)
    ref, ref_lse = oracle.verify_attn(c.q, c.k, c.v, c.cu_seqlens, c.parent, c.n_q)
    err = check_attn(out, ref, c.cfg.dtype, what)
    assert np.abs(lse - ref_lse).max() <= LSE_TOL[c.cfg.dtype], f"{what}: lse"
    return err


def _draft_and_check(sp, oracle, c, what):
    out, lse = run_draft(sp, c)
    ref, ref_lse = oracle.draft_window_attn(c.q, c.k, c.v, c.cu_seqlens, c.text_idx, c.cu_text,
                                            c.window)
    err = check_attn(out, ref, c.cfg.dtype, what)
    assert np.abs(lse - ref_lse).max() <= LSE_TOL[c.cfg.dtype], f"{what}: lse"
    return err


# ------------------------------------------------------------------ the five configurations
@pytest.mark.parametrize("peaked", [False, True])
def test_c1_fp32(sp, oracle, peaked):
    _verify_and_check(sp, oracle, wl.verify_case(wl.C1, 0, peaked=peaked), "C1 verify")
    _draft_and_check(sp, oracle, wl.draft_case(wl.C1, 0, peaked=peaked), "C1 draft")


@pytest.mark.parametrize("peaked", [False, True])
def test_c2_bf16_8k_chain5(sp, oracle, peaked):
    _verify_and_check(sp, oracle, wl.verify_case(wl.C2, 0, peaked=peaked), "C2 verify")
    _draft_and_check(sp, oracle, wl.draft_case(wl.C2, 0, peaked=peaked), "C2 draft")


@pytest.mark.parametrize("peaked", [False, True])
def test_c3_bf16_26k_tree60(sp, oracle, peaked):
    c = wl.verify_case(wl.C3, 0, peaked=peaked)
    assert c.parent is not None and len(c.parent) == 60
    _verify_and_check(sp, oracle, c, "C3 verify")
    _draft_and_check(sp, oracle, wl.draft_case(wl.C3, 0, peaked=peaked), "C3 draft")


@pytest.mark.parametrize("nodes,branching", [(30, (4, 3, 2, 2)), (48, (5, 3, 2, 2, 1)), (25, (5, 3, 2, 2, 1)),
                                             (44, (5, 3, 2, 2, 1)), (16, (4, 2, 1, 1))])
def test_paper_sized_trees_at_26k_context(sp, oracle, nodes, branching):
    """Trees of the sizes the paper's total-depth-width settings give (30, 48 and 25 nodes; 44 and
    16 for the other row-block shapes) at the full 26,112-token context: 4, 6, 3, 5 and 2 tiles of
    64 rows per KV head, run as workgroups of 2+2, 3+3, 3, 3+2 and 2 tiles."""
    parent = wl.pruned_tree(0, nodes, branching)
    c = wl.verify_case(wl.C3, 0, layer=1, n_q=len(parent), parent=parent)
    _verify_and_check(sp, oracle, c, f"tree of {len(parent)} nodes at 26k")


@pytest.mark.parametrize("peaked", [False, True])
def test_c4_bf16_ragged_batch8(sp, oracle, peaked):
    _verify_and_check(sp, oracle, wl.verify_case(wl.C4, 0, peaked=peaked), "C4 verify")
    _draft_and_check(sp, oracle, wl.draft_case(wl.C4, 0, peaked=peaked), "C4 draft")


@pytest.mark.parametrize("layer", [0, 27])
def test_c5_bf16_26k_chain8_layer(sp, oracle, layer):
    """One layer of the benchmarked workload at its full size and launch configuration."""
    _verify_and_check(sp, oracle, wl.verify_case(wl.C5, 0, layer=layer, peaked=(layer == 27)),
                      f"C5 verify layer {layer}")
    if layer == 0:
        _draft_and_check(sp, oracle, wl.draft_case(wl.C5, 0), "C5 draft")


@pytest.mark.parametrize("which", ["C5", "C3", "C4"])
def test_full_size_in_the_benchmarked_kv_layout(sp, oracle, which):
    """bench.py keeps a layer's K and V in one [Hkv, T, 2, d] allocation (head-major, a token's K
    row followed by its V row) and hands the library [T, Hkv, d] views of it: the full-size
    workloads once more in exactly that layout and launch configuration."""
    import torch
    cfg = {"C5": wl.C5, "C3": wl.C3, "C4": wl.C4}[which]
    c = wl.verify_case(cfg, 0, layer=3)
    kv = torch.stack([dev(c.k, "bf16").permute(1, 0, 2), dev(c.v, "bf16").permute(1, 0, 2)], dim=2).contiguous()
    k, v = kv[:, :, 0, :].permute(1, 0, 2), kv[:, :, 1, :].permute(1, 0, 2)
    assert k.stride(0) == 2 * cfg.head_dim and k.stride(1) > k.stride(0)
    par = None if c.parent is None else dev(c.parent)
    out, lse = sp.verify_attn(dev(c.q, "bf16"), k, v, c.cu_seqlens, par, c.n_q)
    torch.cuda.synchronize()
    ref, ref_lse = oracle.verify_attn(c.q, c.k, c.v, c.cu_seqlens, c.parent, c.n_q)
    check_attn(host(out), ref, "bf16", f"{which} in the benchmarked layout")
    assert np.abs(host(lse) - ref_lse).max() <= LSE_TOL["bf16"]


# ------------------------------------------------------------------ shapes, tails, degenerate cases
def _cfg(dtype, Hq, Hkv, d, n_q=4, window=16):
    return wl.Config("T", dtype, Hq, Hkv, d, 1, None, window, n_q, False, 64, 128)


SHAPES = [("f32", 4, 1, 64), ("f32", 8, 2, 128), ("bf16", 8, 2, 64), ("bf16", 28, 4, 128),
          ("bf16", 16, 16, 128), ("bf16", 32, 4, 128)]


@pytest.mark.parametrize("dtype,Hq,Hkv,d", SHAPES)
@pytest.mark.parametrize("L", [0, 1, 31, 33, 257, 1500])
def test_verify_context_lengths(sp, oracle, dtype, Hq, Hkv, d, L):
    """Context lengths around tile boundaries, including an empty context (only the draft rows)."""
    cfg = _cfg(dtype, Hq, Hkv, d)
    lay = (((wl.TEXT, L),),) if L > 0 else (((wl.TEXT, 0),),)
    for n_q in (1, 3, 8):
        c = wl.verify_case(cfg, seed=L + n_q, layouts=lay, n_q=n_q, parent=None)
        _verify_and_check(sp, oracle, c, f"verify {dtype} {Hq}/{Hkv}/{d} L={L} n_q={n_q}")


@pytest.mark.parametrize("lengths,n_q,nodes", [
    ((3000, 3000, 3000), 4, 0),            # 19 splits each: one x range of 24 per (head, sequence)
    ((5200, 4800), 8, 0),                  # 33 + 30 splits in x ranges of 40: padding, rotated XCD order
    ((5000, 4300), 0, 19),                 # 16 + 14 splits, two row blocks of 128 (a tree of 19 nodes)
    ((5200, 4100), 8, 0),                  # 33 + 26 splits: more than a quarter padding -> flat grid
    ((5200, 3900), 0, 19),                 # flat grid with two row blocks
    ((6000, 300, 40, 2500, 10), 5, 0),     # very ragged: flat grid, sequences of a single split
    ((900,), 64, 0),                       # the longest chain the boundary takes (448 rows per KV head)
    (tuple(20 + 37 * i % 300 for i in range(64)), 2, 0),     # the largest batch the boundary takes
])
def test_verify_batches_cover_both_grid_shapes(sp, oracle, lengths, n_q, nodes):
    """Batches of the matrix-core path (bf16, 28/4 heads, d = 128) in the launch shapes the host
    chooses between: per-(head, sequence) x ranges, with and without padding, and the flat grid."""
    cfg = _cfg("bf16", 28, 4, 128)
    lay = tuple(((wl.TEXT, n),) for n in lengths)
    parent = wl.pruned_tree(7, nodes, (4, 3, 2)) if nodes else None
    c = wl.verify_case(cfg, seed=len(lengths) + n_q, layouts=lay,
                       n_q=len(parent) if nodes else n_q, parent=parent)
    _verify_and_check(sp, oracle, c, f"batch {lengths} n_q={c.n_q}")


@pytest.mark.parametrize("Hq,Hkv,nodes", [(4, 4, 0), (4, 4, 33), (32, 2, 0), (32, 2, 40), (32, 2, 64), (16, 1, 21)])
def test_verify_head_groupings(sp, oracle, Hq, Hkv, nodes):
    """Group sizes other than the 7 of the benchmarked model on the matrix-core path (d = 128):
    no grouping at all (one query head per KV head) and 16 query heads per KV head, where a tree
    of 64 nodes is 1,024 rows per KV head (16 tiles of 64 rows, 8 workgroups per split)."""
    cfg = _cfg("bf16", Hq, Hkv, 128)
    parent = wl.pruned_tree(11, nodes, (4, 3, 2, 2, 1, 1)) if nodes else None
    c = wl.verify_case(cfg, seed=Hq + nodes, layouts=(((wl.TEXT, 1300),), ((wl.TEXT, 75),)),
                       n_q=len(parent) if nodes else 7, parent=parent)
    _verify_and_check(sp, oracle, c, f"Hq={Hq} Hkv={Hkv} n_q={c.n_q}")


@pytest.mark.parametrize("seed", range(10))
def test_verify_random_batches(sp, oracle, seed):
    """Seeded random batches on the matrix-core path: 1-7 sequences of 1-4000 context tokens
    (text and visual runs mixed), a chain or a random tree of 1-40 rows, 28/4 or 32/8 heads."""
    rng = np.random.default_rng(9000 + seed)
    Hq, Hkv = ((28, 4), (32, 8))[seed % 2]
    cfg = _cfg("bf16", Hq, Hkv, 128)
    B = int(rng.integers(1, 8))
    lay = []
    for _ in range(B):
        n = int(rng.integers(1, 4001)) if rng.random() < 0.8 else int(rng.integers(1, 40))
        cut = int(rng.integers(0, n + 1))
        lay.append(tuple(seg for seg in ((wl.VISUAL, cut), (wl.TEXT, n - cut)) if seg[1] > 0))
    if rng.random() < 0.5:
        n_q, parent = int(rng.integers(1, 17)), None
    else:
        nodes = int(rng.integers(2, 41))
        parent = wl.pruned_tree(seed, nodes, (4, 3, 2, 2, 1, 1))
        n_q = len(parent)
    c = wl.verify_case(cfg, seed=seed, layouts=tuple(lay), n_q=n_q, parent=parent)
    _verify_and_check(sp, oracle, c, f"random batch {seed}: B={B} n_q={n_q} tree={parent is not None}")


@pytest.mark.parametrize("dtype,Hq,Hkv,d", [("f32", 4, 1, 64), ("bf16", 28, 4, 128)])
@pytest.mark.parametrize("n_q", [5, 33, 64])
def test_verify_arbitrary_random_trees(sp, oracle, dtype, Hq, Hkv, d, n_q):
    """Trees of any shape (every parent drawn uniformly among the root and the earlier nodes: long
    chains, wide stars and everything between, up to the 64 nodes the boundary takes), one per
    sequence, against short and empty contexts, where the draft rows' mask decides most of the
    result."""
    cfg = _cfg(dtype, Hq, Hkv, d)
    for seed in range(3):
        rng = np.random.default_rng(1000 * n_q + seed)
        lengths = (int(rng.integers(0, 400)), int(rng.integers(0, 60)), 0)
        trees = np.stack([np.array([int(rng.integers(-1, i)) for i in range(n_q)], dtype=np.int32)
                          for _ in lengths])
        lay = tuple(((wl.TEXT, n),) for n in lengths)
        c = wl.verify_case(cfg, seed=seed, layouts=lay, n_q=n_q, parent=trees, peaked=(seed == 1))
        _verify_and_check(sp, oracle, c, f"random trees {dtype} n_q={n_q} seed {seed} {lengths}")


@pytest.mark.parametrize("dtype,Hq,Hkv,d", [("f32", 4, 1, 64), ("bf16", 28, 4, 128)])
def test_verify_trees(sp, oracle, dtype, Hq, Hkv, d):
    cfg = _cfg(dtype, Hq, Hkv, d)
    lay = (((wl.TEXT, 700),), ((wl.TEXT, 90),))
    trees = [wl.chain_parent(7), np.full(5, -1, dtype=np.int32),
             wl.pruned_tree(1, 25, (4, 2, 2, 1, 1)), wl.pruned_tree(2, 30, (8, 2, 1, 1)),
             wl.pruned_tree(3, 48, (10, 2, 2, 1, 1)), wl.pruned_tree(4, 64, (4, 4, 2, 2, 1, 1)),
             # 70 and 133 rows per KV head at 28/4 heads: a 128-row workgroup whose second row
             # tile is nearly empty, and a second workgroup with five rows
             wl.pruned_tree(5, 10, (3, 2, 2)), wl.pruned_tree(6, 19, (4, 3, 2))]
    for ti, parent in enumerate(trees):
        c = wl.verify_case(cfg, seed=50 + ti, layouts=lay, n_q=len(parent), parent=parent)
        _verify_and_check(sp, oracle, c, f"tree {ti} ({len(parent)} nodes) {dtype}")
    # a chain given as a tree gives bit-identical output to parent = NULL
    c = wl.verify_case(cfg, seed=60, layouts=lay, n_q=6, parent=None)
    a, _ = run_verify(sp, c)
    c.parent = wl.chain_parent(6)
    b, _ = run_verify(sp, c)
    np.testing.assert_array_equal(a, b)


@pytest.mark.parametrize("dtype,Hq,Hkv,d", [("f32", 4, 1, 64), ("bf16", 28, 4, 128), ("bf16", 8, 2, 64)])
def test_verify_one_tree_per_sequence(sp, oracle, dtype, Hq, Hkv, d):
    """A batch in which every sequence grew a draft tree of its own (dynamic trees differ between
    requests): parent is [B, n_q], and each sequence's rows follow its own ancestor sets.  Checked
    against the oracle run sequence by sequence with that sequence's tree, on both kernel paths,
    both grid shapes of the matrix-core path (even and very uneven lengths) and through the
    entry point on the library's static scratch."""
    import torch
    cfg = _cfg(dtype, Hq, Hkv, d)
    for lengths, nodes in (((1500, 1400, 1450), 30), ((2600, 90, 700, 5), 48), ((300, 200), 7)):
        branching = (4, 3, 2, 2, 1, 1) if nodes > 8 else (3, 2)
        trees = np.stack([wl.pruned_tree(100 + i, nodes, branching) for i in range(len(lengths))])
        n_q = trees.shape[1]
        assert any(not np.array_equal(trees[0], t) for t in trees[1:]), "the trees must differ"
        lay = tuple(((wl.TEXT, n),) for n in lengths)
        c = wl.verify_case(cfg, seed=nodes, layouts=lay, n_q=n_q, parent=trees)
        _verify_and_check(sp, oracle, c, f"per-sequence trees {dtype} {lengths} n_q={n_q}")
        # the same call with every sequence on tree 0 must differ (the per-sequence trees are used)
        c0 = wl.verify_case(cfg, seed=nodes, layouts=lay, n_q=n_q, parent=trees[0])
        a, _ = run_verify(sp, c)
        b, _ = run_verify(sp, c0)
        np.testing.assert_array_equal(a[:n_q], b[:n_q])          # sequence 0: same tree, same bits
        assert not np.array_equal(a[n_q:], b[n_q:])
        if dtype == "bf16" and d == 128:
            q, k, v = dev(c.q, dtype), dev(c.k, dtype), dev(c.v, dtype)
            out = torch.empty_like(q)
            sp.verify_attn_static(q, k, v, c.cu_seqlens, dev(trees), n_q, out)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(host(out), a)


@pytest.mark.parametrize("dtype,Hq,Hkv,d", SHAPES)
def test_draft_windows_and_layouts(sp, oracle, dtype, Hq, Hkv, d):
    cfg = _cfg(dtype, Hq, Hkv, d)
    lays = (((wl.TEXT, 5), (wl.VISUAL, 400), (wl.TEXT, 3), (wl.VISUAL, 170), (wl.TEXT, 90)),
            ((wl.VISUAL, 300), (wl.TEXT, 1)),
            ((wl.TEXT, 700),))
    for window in (1, 2, 63, 64, 65, 98, 512, 4096):
        c = wl.draft_case(cfg, seed=window, layouts=lays, window=window)
        _draft_and_check(sp, oracle, c, f"draft {dtype} {Hq}/{Hkv}/{d} W={window}")


def test_draft_ignores_poisoned_visual_kv(sp, oracle):
    """NaN in every visual K/V slot: the kernel never addresses them."""
    c = wl.draft_case(wl.C2, 1)
    ref, _ = oracle.draft_window_attn(c.q, c.k, c.v, c.cu_seqlens, c.text_idx, c.cu_text, c.window)
    vis = np.flatnonzero(c.types[0] == wl.VISUAL)
    c.k[vis] = np.nan
    c.v[vis] = np.nan
    out, _ = run_draft(sp, c)
    check_attn(out, ref, "bf16", "poisoned visual KV")


def test_strided_kv_and_explicit_scale(sp, oracle):
    """K/V given as slices of a wider buffer (non-default strides) and a caller-chosen scale."""
    import torch
    from gpu_util import dev, host
    cfg = _cfg("bf16", 28, 4, 128)
    c = wl.verify_case(cfg, seed=5, layouts=(((wl.TEXT, 900),),), n_q=5, parent=None)
    T = c.k.shape[0]
    wide_k = torch.zeros(T, 6, 160, dtype=torch.bfloat16, device="cuda")
    wide_v = torch.zeros_like(wide_k)
    wide_k[:, 1:5, 16:144] = dev(c.k, "bf16")
    wide_v[:, 1:5, 16:144] = dev(c.v, "bf16")
    out, _ = sp.verify_attn(dev(c.q, "bf16"), wide_k[:, 1:5, 16:144], wide_v[:, 1:5, 16:144],
                            c.cu_seqlens, None, 5, scale=0.05)
    torch.cuda.synchronize()
    ref, _ = oracle.verify_attn(c.q, c.k, c.v, c.cu_seqlens, None, 5, scale=0.05)
    check_attn(host(out), ref, "bf16", "strided kv")


@pytest.mark.parametrize("interleaved", [False, True])
def test_head_major_kv_layout(sp, oracle, interleaved):
    """K/V stored [Hkv, T, d] (a head's tokens contiguous) and passed as a [T, Hkv, d] view: same
    results as the token-major layout, for the verification and the draft attention, chain and
    tree, matrix-core and plain-ALU kernels.  Interleaved: one [Hkv, T, 2, d] allocation, a token's
    K row followed by its V row (k and v are views into it with a token stride of 2 d)."""
    import torch
    for dtype, Hq, Hkv, d in (("bf16", 28, 4, 128), ("f32", 4, 2, 64)):
        cfg = _cfg(dtype, Hq, Hkv, d)
        lay = (((wl.TEXT, 50), (wl.VISUAL, 1100), (wl.TEXT, 77)), ((wl.VISUAL, 300), (wl.TEXT, 45)))

        def hm_pair(kh, vh):
            if not interleaved:
                hm = lambda x: dev(x, dtype).permute(1, 0, 2).contiguous().permute(1, 0, 2)   # noqa: E731
                return hm(kh), hm(vh)
            kv = torch.stack([dev(kh, dtype).permute(1, 0, 2), dev(vh, dtype).permute(1, 0, 2)], dim=2).contiguous()
            return kv[:, :, 0, :].permute(1, 0, 2), kv[:, :, 1, :].permute(1, 0, 2)
        for parent in (None, wl.pruned_tree(1, 25, (4, 2, 2, 1, 1))):
            n_q = 6 if parent is None else len(parent)
            c = wl.verify_case(cfg, seed=77, layouts=lay, n_q=n_q, parent=parent)
            k, v = hm_pair(c.k, c.v)
            assert k.stride(1) > k.stride(0) and k.stride(0) == (2 * d if interleaved else d)
            par = None if parent is None else dev(parent)
            out, lse = sp.verify_attn(dev(c.q, dtype), k, v, c.cu_seqlens, par, n_q)
            torch.cuda.synchronize()
            ref, ref_lse = oracle.verify_attn(c.q, c.k, c.v, c.cu_seqlens, parent, n_q)
            check_attn(host(out), ref, dtype, f"head-major verify {dtype} n_q={n_q}")
        dc = wl.draft_case(cfg, seed=78, layouts=lay)
        k, v = hm_pair(dc.k, dc.v)
        out, _ = sp.draft_window_attn(dev(dc.q, dtype), k, v, dc.cu_seqlens, dev(dc.text_idx), dc.cu_text,
                                      dc.window)
        torch.cuda.synchronize()
        ref, _ = oracle.draft_window_attn(dc.q, dc.k, dc.v, dc.cu_seqlens, dc.text_idx, dc.cu_text, dc.window)
        check_attn(host(out), ref, dtype, f"head-major draft {dtype}")


def test_kv_span_of_2_gib_takes_the_plain_alu_kernels(sp, oracle):
    """bf16, d = 128, but the K/V rows lie 8 MiB apart in one 2.2 GB allocation: a sequence's rows
    can then no longer be addressed by the 32-bit offsets of the matrix-core kernel, and the call
    (and its workspace query) fall back to the plain-ALU partial and combine kernels in bf16 with
    head_dim 128 and 64-bit addressing.  Chain and a small tree, two sequences."""
    import torch
    cfg = _cfg("bf16", 28, 4, 128)
    stride = 1 << 22                              # elements between consecutive tokens
    lay = (((wl.TEXT, 20), (wl.VISUAL, 200), (wl.TEXT, 37)), ((wl.TEXT, 3),))
    for parent in (None, wl.pruned_tree(3, 9, (3, 2, 1))):
        n_q = 6 if parent is None else len(parent)
        c = wl.verify_case(cfg, seed=31 + n_q, layouts=lay, n_q=n_q, parent=parent)
        T = c.k.shape[0]
        assert T * stride * 2 >= 2 ** 31, "the case must span 2 GiB to leave the matrix-core path"
        buf = torch.empty(T * stride, dtype=torch.bfloat16, device="cuda").view(T, stride)
        k = buf[:, :512].view(T, 4, 128)
        v = buf[:, stride // 2:stride // 2 + 512].view(T, 4, 128)
        k.copy_(dev(c.k, "bf16"))
        v.copy_(dev(c.v, "bf16"))
        q = dev(c.q, "bf16")
        par = None if parent is None else dev(parent)
        out, lse = sp.verify_attn(q, k, v, c.cu_seqlens, par, n_q)
        torch.cuda.synchronize()
        ref, ref_lse = oracle.verify_attn(c.q, c.k, c.v, c.cu_seqlens, parent, n_q)
        check_attn(host(out), ref, "bf16", f"2 GiB span, n_q={n_q}")
        assert np.abs(host(lse) - ref_lse).max() <= LSE_TOL["bf16"]
        # the same rows packed densely run on the matrix cores: a different workspace layout
        # (fp16 tiles per 64-row block against fp32 rows per split), so the two queries differ
        dense_k = dev(c.k, "bf16")
        need_far = sp.verify_attn_workspace_bytes(q, k, v, 2, n_q, T)
        need_dense = sp.verify_attn_workspace_bytes(q, dense_k, dense_k, 2, n_q, T)
        assert need_far != need_dense and need_far > 0
        del buf, k, v
        torch.cuda.empty_cache()


def test_large_v_does_not_overflow_the_split_partials(sp, oracle):
    """The matrix-core path keeps the split outputs as fp16 with a per-row power-of-two scale:
    V of magnitude 2^20 and 2^100 (far outside fp16) must come out as exactly that multiple of
    the ordinary result, with the usual relative error."""
    cfg = _cfg("bf16", 28, 4, 128)
    lay = (((wl.TEXT, 50), (wl.VISUAL, 2100), (wl.TEXT, 77)),)
    c = wl.verify_case(cfg, seed=91, layouts=lay, n_q=8, parent=None)
    base, _ = run_verify(sp, c)
    for p2 in (20, 100):
        c2 = wl.verify_case(cfg, seed=91, layouts=lay, n_q=8, parent=None)
        c2.v = (c2.v.astype(np.float64) * 2.0 ** p2).astype(np.float32)        # exact in bf16
        out, _ = run_verify(sp, c2)
        assert np.all(np.isfinite(out))
        ref, _ = oracle.verify_attn(c2.q, c2.k, c2.v, c2.cu_seqlens, None, 8)
        scale = np.abs(ref).max()
        assert np.abs(out - ref).max() <= 2e-2 * scale, f"2^{p2}"
        # same bits as the unscaled run, shifted by the exponent
        np.testing.assert_array_equal(out, base * 2.0 ** p2)


def test_argument_errors(sp):
    import torch
    from gpu_util import dev
    c = wl.verify_case(_cfg("bf16", 28, 4, 128), seed=6, layouts=(((wl.TEXT, 100),),), n_q=3,
                       parent=None)
    q, k, v = dev(c.q, "bf16"), dev(c.k, "bf16"), dev(c.v, "bf16")
    with pytest.raises(sp.SparrowError) as e:   # workspace too small
        sp.verify_attn(q, k, v, c.cu_seqlens, None, 3,
                       workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.code == -3
    with pytest.raises(sp.SparrowError) as e:   # a sequence shorter than n_q
        sp.verify_attn(q, k, v, np.array([0, 2], dtype=np.int32), None, 3)
    assert e.value.code == -1
    d = wl.draft_case(_cfg("bf16", 28, 4, 128), seed=7, layouts=(((wl.TEXT, 100),),))
    with pytest.raises(sp.SparrowError) as e:   # empty text domain
        sp.draft_window_attn(dev(d.q, "bf16"), dev(d.k, "bf16"), dev(d.v, "bf16"), d.cu_seqlens,
                             dev(d.text_idx), np.array([0, 0], dtype=np.int32), 8)
    assert e.value.code == -1 and "text" in str(e.value)
    with pytest.raises(sp.SparrowError):        # window <= 0
        sp.draft_window_attn(dev(d.q, "bf16"), dev(d.k, "bf16"), dev(d.v, "bf16"), d.cu_seqlens,
                             dev(d.text_idx), d.cu_text, 0)
    # B = 0 / n_q = 0 are no-ops
    out, _ = sp.verify_attn(q[:0], k, v, np.array([0, 103], dtype=np.int32), None, 0)
    assert out.numel() == 0
