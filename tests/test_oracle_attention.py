"""Pins for the attention oracles (CPU only).

The oracle is checked against things other than itself: torch's CPU fp64
scaled_dot_product_attention with an explicit dense mask, scipy's
softmax/logsumexp, closed forms, and invariants of the definitions (VATA,
Eq. 2: attention closed within the text domain; verification: all context plus
ancestors-or-self among the draft rows)."""
import numpy as np
import pytest
import torch
from scipy.special import logsumexp, softmax

import workloads as wl


def sdpa_dense(q, k, v, mask, scale):
    """q [R,Hq,d], k/v [T,Hkv,d], mask bool [R,T] -> [R,Hq,d] via torch SDPA (fp64)."""
    Hq, Hkv = q.shape[1], k.shape[1]
    g = Hq // Hkv
    qt = torch.from_numpy(np.ascontiguousarray(q, dtype=np.float64)).permute(1, 0, 2)[None]
    kt = torch.from_numpy(np.ascontiguousarray(k, dtype=np.float64)).permute(1, 0, 2)
    vt = torch.from_numpy(np.ascontiguousarray(v, dtype=np.float64)).permute(1, 0, 2)
    kt = kt.repeat_interleave(g, dim=0)[None]
    vt = vt.repeat_interleave(g, dim=0)[None]
    m = torch.from_numpy(mask)[None, None]
    o = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, attn_mask=m, scale=scale)
    return o[0].permute(1, 0, 2).numpy()


def small_cfg(Hq=4, Hkv=2, d=16, dtype="f32"):
    return wl.Config("S", dtype, Hq, Hkv, d, 1, None, 8, 3, False, 32, 64)


LAYOUTS = (((wl.TEXT, 5), (wl.VISUAL, 40), (wl.TEXT, 3), (wl.VISUAL, 17), (wl.TEXT, 9)),
           ((wl.VISUAL, 30), (wl.TEXT, 6)))


# ---------------------------------------------------------------- draft (O1)
@pytest.mark.parametrize("window", [1, 4, 9, 12, 17, 1000])
def test_draft_matches_torch_sdpa_dense_mask(oracle, window):
    cfg = small_cfg()
    c = wl.draft_case(cfg, seed=3, layouts=LAYOUTS, window=window)
    out, lse = oracle.draft_window_attn(c.q, c.k, c.v, c.cu_seqlens, c.text_idx, c.cu_text, window)
    scale = 1.0 / np.sqrt(cfg.head_dim)
    for b in range(2):
        lo, hi = c.cu_seqlens[b], c.cu_seqlens[b + 1]
        tpos = np.flatnonzero(c.types[b] == wl.TEXT)
        sel = tpos[-window:]
        mask = np.zeros((1, hi - lo), dtype=bool)
        mask[0, sel] = True
        ref = sdpa_dense(c.q[b:b + 1], c.k[lo:hi], c.v[lo:hi], mask, scale)
        np.testing.assert_allclose(out[b], ref[0], rtol=0, atol=1e-13)
        # lse by scipy on independently formed scores
        s = np.einsum("hx,thx->ht", c.q[b].astype(np.float64).reshape(cfg.n_kv_heads, -1, cfg.head_dim)
                      .reshape(cfg.n_q_heads, cfg.head_dim),
                      np.repeat(c.k[lo:hi].astype(np.float64), cfg.group, axis=1)[sel]) * scale
        np.testing.assert_allclose(lse[b], logsumexp(s, axis=1), rtol=0, atol=1e-13)


def test_draft_never_reads_visual_slots(oracle):
    """Poison every visual K/V slot with NaN/Inf: the output must not change
    (the visual KV cache is discarded for the draft)."""
    cfg = small_cfg()
    c = wl.draft_case(cfg, seed=4, layouts=LAYOUTS, window=1000)
    ref, _ = oracle.draft_window_attn(c.q, c.k, c.v, c.cu_seqlens, c.text_idx, c.cu_text, 1000)
    k, v = c.k.copy(), c.v.copy()
    for b in range(2):
        vis = np.flatnonzero(c.types[b] == wl.VISUAL) + c.cu_seqlens[b]
        k[vis] = np.nan
        v[vis] = np.inf
    out, _ = oracle.draft_window_attn(c.q, k, v, c.cu_seqlens, c.text_idx, c.cu_text, 1000)
    assert np.isfinite(out).all()
    np.testing.assert_array_equal(out, ref)


def test_draft_all_text_full_window_is_causal_decode(oracle):
    """All positions text and W >= L: the last position's causal attention."""
    cfg = small_cfg(Hq=6, Hkv=2, d=8)
    L = 37
    lay = (((wl.TEXT, L),),)
    c = wl.draft_case(cfg, seed=5, layouts=lay, window=L + 5)
    out, _ = oracle.draft_window_attn(c.q, c.k, c.v, c.cu_seqlens, c.text_idx, c.cu_text, L + 5)
    # full causal self-attention over L rows with torch's is_causal; take the last row
    g = cfg.group
    qfull = np.zeros((L, cfg.n_q_heads, cfg.head_dim))
    qfull[-1] = c.q[0]
    qt = torch.from_numpy(qfull).permute(1, 0, 2)[None]
    kt = torch.from_numpy(c.k.astype(np.float64)).permute(1, 0, 2).repeat_interleave(g, 0)[None]
    vt = torch.from_numpy(c.v.astype(np.float64)).permute(1, 0, 2).repeat_interleave(g, 0)[None]
    o = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, is_causal=True)
    np.testing.assert_allclose(out[0], o[0, :, -1].numpy(), rtol=0, atol=1e-13)


def test_draft_closed_forms(oracle):
    cfg = small_cfg()
    c = wl.draft_case(cfg, seed=6, layouts=LAYOUTS[:1], window=10)
    tpos = np.flatnonzero(c.types[0] == wl.TEXT)[-10:]
    # V constant -> output is that constant
    v = np.full_like(c.v, 0.375)
    out, _ = oracle.draft_window_attn(c.q, c.k, v, c.cu_seqlens, c.text_idx, c.cu_text, 10)
    np.testing.assert_allclose(out, 0.375, rtol=0, atol=1e-15)
    # K zero -> uniform weights -> mean of the window's V rows, lse = log(W)
    out, lse = oracle.draft_window_attn(c.q, np.zeros_like(c.k), c.v, c.cu_seqlens, c.text_idx,
                                        c.cu_text, 10)
    mean = c.v[tpos].astype(np.float64).mean(axis=0)  # [Hkv, d]
    np.testing.assert_allclose(out[0], np.repeat(mean, cfg.group, axis=0), rtol=0, atol=1e-14)
    np.testing.assert_allclose(lse, np.log(10.0), rtol=0, atol=1e-14)
    # one key hugely aligned with q (only for head 0) -> output -> that V row
    k = np.zeros_like(c.k)
    j = tpos[3]
    k[j, 0] = 200.0 * c.q[0, 0] / np.linalg.norm(c.q[0, 0])
    out, _ = oracle.draft_window_attn(c.q, k, c.v, c.cu_seqlens, c.text_idx, c.cu_text, 10)
    np.testing.assert_allclose(out[0, 0], c.v[j, 0], rtol=0, atol=1e-12)


def test_draft_window_recurrence(oracle):
    """W and W+1 differ by exactly one extra key: merge it by hand via lse."""
    cfg = small_cfg()
    c = wl.draft_case(cfg, seed=7, layouts=LAYOUTS[:1])
    scale = 1.0 / np.sqrt(cfg.head_dim)
    tpos = np.flatnonzero(c.types[0] == wl.TEXT)
    for W in (1, 5, 9):
        o0, l0 = oracle.draft_window_attn(c.q, c.k, c.v, c.cu_seqlens, c.text_idx, c.cu_text, W)
        o1, l1 = oracle.draft_window_attn(c.q, c.k, c.v, c.cu_seqlens, c.text_idx, c.cu_text, W + 1)
        extra = tpos[-(W + 1)]
        for h in range(cfg.n_q_heads):
            kv = h // cfg.group
            s = scale * float(c.q[0, h].astype(np.float64) @ c.k[extra, kv].astype(np.float64))
            lnew = np.logaddexp(l0[0, h], s)
            onew = (np.exp(l0[0, h] - lnew) * o0[0, h]
                    + np.exp(s - lnew) * c.v[extra, kv].astype(np.float64))
            np.testing.assert_allclose(l1[0, h], lnew, rtol=0, atol=1e-13)
            np.testing.assert_allclose(o1[0, h], onew, rtol=0, atol=1e-13)


def test_draft_scale_argument(oracle):
    """scale is an explicit parameter: the literal reading of Eq. 2 (d = model
    hidden size) is one argument away and differs from the per-head reading."""
    cfg = small_cfg()
    c = wl.draft_case(cfg, seed=8, layouts=LAYOUTS[:1], window=9)
    a, _ = oracle.draft_window_attn(c.q, c.k, c.v, c.cu_seqlens, c.text_idx, c.cu_text, 9)
    b, _ = oracle.draft_window_attn(c.q, c.k, c.v, c.cu_seqlens, c.text_idx, c.cu_text, 9,
                                    scale=1.0 / np.sqrt(cfg.head_dim))
    np.testing.assert_array_equal(a, b)
    h = cfg.n_q_heads * cfg.head_dim
    lit, _ = oracle.draft_window_attn(c.q, c.k, c.v, c.cu_seqlens, c.text_idx, c.cu_text, 9,
                                      scale=1.0 / np.sqrt(h))
    q2 = c.q.astype(np.float64) * np.sqrt(cfg.head_dim / h)
    viaq, _ = oracle.draft_window_attn(q2, c.k, c.v, c.cu_seqlens, c.text_idx, c.cu_text, 9)
    np.testing.assert_allclose(lit, viaq, rtol=0, atol=1e-13)
    assert np.abs(lit - a).max() > 1e-3


def test_draft_rejects_empty_text_domain(oracle):
    cfg = small_cfg()
    c = wl.draft_case(cfg, seed=9, layouts=LAYOUTS, window=4)
    cu_text = c.cu_text.copy()
    cu_text[1] = 0  # sequence 0 has no text position
    with pytest.raises(ValueError):
        oracle.draft_window_attn(c.q, c.k, c.v, c.cu_seqlens, c.text_idx, cu_text, 4)
    with pytest.raises(ValueError):
        oracle.draft_window_attn(c.q, c.k, c.v, c.cu_seqlens, c.text_idx, c.cu_text, 0)


# --------------------------------------------------------------- verify (O2)
def dense_verify_mask(L, n_q, parent):
    mask = np.zeros((n_q, L + n_q), dtype=bool)
    mask[:, :L] = True
    for i in range(n_q):
        a = i
        while a >= 0:
            mask[i, L + a] = True
            a = (a - 1) if parent is None else int(parent[a])
    return mask


TREES = [None,
         np.array([-1, 0, 1, 2, 3], dtype=np.int32),          # chain written as a tree
         np.array([-1, -1, 0, 0, 1, 3, 3, 6], dtype=np.int32),
         np.array([-1, -1, -1, -1], dtype=np.int32),          # four roots
         wl.pruned_tree(11, 25, (4, 2, 2, 1, 1))]


@pytest.mark.parametrize("ti", range(len(TREES)))
def test_verify_matches_torch_sdpa_dense_mask(oracle, ti):
    parent = TREES[ti]
    n_q = 5 if parent is None else len(parent)
    cfg = small_cfg(Hq=6, Hkv=2, d=16)
    c = wl.verify_case(cfg, seed=20 + ti, layouts=LAYOUTS, n_q=n_q, parent=parent)
    out, lse = oracle.verify_attn(c.q, c.k, c.v, c.cu_seqlens, parent, n_q)
    scale = 1.0 / np.sqrt(cfg.head_dim)
    for b in range(2):
        lo, hi = c.cu_seqlens[b], c.cu_seqlens[b + 1]
        L = hi - lo - n_q
        mask = dense_verify_mask(L, n_q, parent)
        ref = sdpa_dense(c.q[b * n_q:(b + 1) * n_q], c.k[lo:hi], c.v[lo:hi], mask, scale)
        np.testing.assert_allclose(out[b * n_q:(b + 1) * n_q], ref, rtol=0, atol=1e-13)
        # probabilities sum to 1 <=> exp(s - lse) sums to 1 (scores formed independently)
        kk = np.repeat(c.k[lo:hi].astype(np.float64), cfg.group, axis=1)
        s = np.einsum("rhx,thx->rht", c.q[b * n_q:(b + 1) * n_q].astype(np.float64), kk) * scale
        s = np.where(mask[:, None, :], s, -np.inf)
        np.testing.assert_allclose(lse[b * n_q:(b + 1) * n_q], logsumexp(s, axis=2), atol=1e-13,
                                   rtol=0)
        p = softmax(s, axis=2)
        np.testing.assert_allclose(p.sum(axis=2), 1.0, atol=1e-12, rtol=0)


def test_verify_chain_tree_equals_chain(oracle):
    cfg = small_cfg()
    n_q = 6
    c = wl.verify_case(cfg, seed=31, layouts=LAYOUTS, n_q=n_q, parent=None)
    a, la = oracle.verify_attn(c.q, c.k, c.v, c.cu_seqlens, None, n_q)
    b, lb = oracle.verify_attn(c.q, c.k, c.v, c.cu_seqlens, wl.chain_parent(n_q), n_q)
    np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(la, lb)


def test_verify_single_row_is_decode(oracle):
    """n_q = 1: one-token decode over L+1 rows == draft oracle with an all-text
    index and a window covering everything."""
    cfg = small_cfg()
    c = wl.verify_case(cfg, seed=32, layouts=LAYOUTS, n_q=1, parent=None)
    out, lse = oracle.verify_attn(c.q, c.k, c.v, c.cu_seqlens, None, 1)
    lens = np.diff(c.cu_seqlens)
    text_idx = np.concatenate([np.arange(n, dtype=np.int32) for n in lens])
    cu_text = c.cu_seqlens.copy()
    o2, l2 = oracle.draft_window_attn(c.q, c.k, c.v, c.cu_seqlens, text_idx, cu_text,
                                      int(lens.max()) + 1)
    np.testing.assert_allclose(out, o2, rtol=0, atol=1e-15)
    np.testing.assert_allclose(lse, l2, rtol=0, atol=1e-15)


def test_verify_tree_per_path_decomposition(oracle):
    """Row i of a tree equals the last row of a chain verification of the
    root->i path (K/V rows of the path gathered in order)."""
    cfg = small_cfg()
    parent = wl.pruned_tree(12, 20, (3, 2, 2, 2))
    n_q = len(parent)
    lay = LAYOUTS[:1]
    c = wl.verify_case(cfg, seed=33, layouts=lay, n_q=n_q, parent=parent)
    out, lse = oracle.verify_attn(c.q, c.k, c.v, c.cu_seqlens, parent, n_q)
    L = c.cu_seqlens[1] - n_q
    for i in range(n_q):
        path = []
        a = i
        while a >= 0:
            path.append(a)
            a = int(parent[a])
        path = path[::-1]
        rows = np.concatenate([np.arange(L), L + np.array(path)])
        kc, vc = c.k[rows], c.v[rows]
        qc = c.q[path]
        cu = np.array([0, L + len(path)], dtype=np.int32)
        oc, lc = oracle.verify_attn(qc, kc, vc, cu, None, len(path))
        np.testing.assert_allclose(out[i], oc[-1], rtol=0, atol=1e-14)
        np.testing.assert_allclose(lse[i], lc[-1], rtol=0, atol=1e-14)


def test_verify_context_permutation_invariance(oracle):
    cfg = small_cfg()
    n_q = 4
    lay = LAYOUTS[:1]
    c = wl.verify_case(cfg, seed=34, layouts=lay, n_q=n_q, parent=None)
    out, _ = oracle.verify_attn(c.q, c.k, c.v, c.cu_seqlens, None, n_q)
    L = c.cu_seqlens[1] - n_q
    perm = np.concatenate([np.random.default_rng(0).permutation(L), L + np.arange(n_q)])
    o2, _ = oracle.verify_attn(c.q, c.k[perm], c.v[perm], c.cu_seqlens, None, n_q)
    np.testing.assert_allclose(out, o2, rtol=0, atol=1e-14)


def test_verify_split_and_merge_algebra(oracle):
    """Partition the context, attend to each part, merge (m, l, o) partials:
    reproduces the unsplit result (the algebra the GPU split-context path uses,
    here checked in fp64 on the oracle alone)."""
    cfg = small_cfg()
    lay = (((wl.TEXT, 50),),)
    c = wl.verify_case(cfg, seed=35, layouts=lay, n_q=1, parent=None)
    out, lse = oracle.verify_attn(c.q, c.k, c.v, c.cu_seqlens, None, 1)
    cuts = [0, 7, 8, 30, 51]
    parts = []
    for a, b in zip(cuts[:-1], cuts[1:]):
        n = b - a
        # each part as its own one-row decode: context n-1 rows + 1 "draft" row
        cu = np.array([0, n], dtype=np.int32)
        parts.append(oracle.verify_attn(c.q, c.k[a:b], c.v[a:b], cu, None, 1))
    lses = np.stack([p[1] for p in parts])          # [S, 1, Hq]
    outs = np.stack([p[0] for p in parts])          # [S, 1, Hq, d]
    tot = logsumexp(lses, axis=0)
    w = np.exp(lses - tot[None])
    merged = (w[..., None] * outs).sum(axis=0)
    np.testing.assert_allclose(tot, lse, rtol=0, atol=1e-13)
    np.testing.assert_allclose(merged, out, rtol=0, atol=1e-13)


def test_verify_gqa_equals_replicated_mha(oracle):
    cfg = small_cfg(Hq=6, Hkv=2, d=8)
    n_q = 3
    c = wl.verify_case(cfg, seed=36, layouts=LAYOUTS, n_q=n_q, parent=None)
    a, _ = oracle.verify_attn(c.q, c.k, c.v, c.cu_seqlens, None, n_q)
    krep = np.repeat(c.k, cfg.group, axis=1)
    vrep = np.repeat(c.v, cfg.group, axis=1)
    b, _ = oracle.verify_attn(c.q, krep, vrep, c.cu_seqlens, None, n_q)
    np.testing.assert_array_equal(a, b)


def test_verify_rejects_bad_parent(oracle):
    cfg = small_cfg()
    c = wl.verify_case(cfg, seed=37, layouts=LAYOUTS[:1], n_q=3, parent=None)
    with pytest.raises(ValueError):
        oracle.verify_attn(c.q, c.k, c.v, c.cu_seqlens, np.array([-1, 1, 0], dtype=np.int32), 3)


def test_c1_config_shapes_and_full_size_pin(oracle):
    """C1 at its real size against torch SDPA (both attention oracles)."""
    cfg = wl.C1
    d = wl.draft_case(cfg, seed=0)
    assert d.k.shape == (512, 1, 64) and d.q.shape == (1, 4, 64)
    assert list(d.text_idx[:16]) == list(range(16)) and list(d.text_idx[16:]) == list(range(464, 512))
    out, _ = oracle.draft_window_attn(d.q, d.k, d.v, d.cu_seqlens, d.text_idx, d.cu_text, cfg.window)
    mask = np.zeros((1, 512), dtype=bool)
    mask[0, 480:512] = True
    ref = sdpa_dense(d.q, d.k, d.v, mask, 1.0 / 8.0)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-13)
    v = wl.verify_case(cfg, seed=0)
    assert v.k.shape == (516, 1, 64) and v.q.shape == (4, 4, 64) and v.parent is None
    out, _ = oracle.verify_attn(v.q, v.k, v.v, v.cu_seqlens, None, 4)
    ref = sdpa_dense(v.q, v.k, v.v, dense_verify_mask(512, 4, None), 1.0 / 8.0)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-13)


def test_one_tree_per_sequence_is_the_per_sequence_result(oracle):
    """parent [B, n_q]: sequence b is verified with tree b.  Equal rows reproduce the shared-tree
    call bit for bit; different rows reproduce, sequence by sequence, a single-sequence call with
    that tree (and differ from the shared-tree result where the trees differ)."""
    cfg = wl.Config("T", "f32", 4, 2, 64, 1, None, 8, 4, False, 64, 128)
    lay = (((wl.TEXT, 37),), ((wl.TEXT, 5),), ((wl.TEXT, 60),))
    trees = np.stack([wl.pruned_tree(i, 9, (3, 2, 2)) for i in range(3)])
    n_q = trees.shape[1]
    c = wl.verify_case(cfg, seed=4, layouts=lay, n_q=n_q, parent=None)
    shared, shared_lse = oracle.verify_attn(c.q, c.k, c.v, c.cu_seqlens, trees[0], n_q)
    same, same_lse = oracle.verify_attn(c.q, c.k, c.v, c.cu_seqlens, np.stack([trees[0]] * 3), n_q)
    np.testing.assert_array_equal(shared, same)
    np.testing.assert_array_equal(shared_lse, same_lse)
    own, _ = oracle.verify_attn(c.q, c.k, c.v, c.cu_seqlens, trees, n_q)
    cu = c.cu_seqlens
    for b in range(3):
        one, _ = oracle.verify_attn(c.q[b * n_q:(b + 1) * n_q], c.k[cu[b]:cu[b + 1]], c.v[cu[b]:cu[b + 1]],
                                    [0, cu[b + 1] - cu[b]], trees[b], n_q)
        np.testing.assert_array_equal(own[b * n_q:(b + 1) * n_q], one)
    assert not np.array_equal(own[n_q:], shared[n_q:])
