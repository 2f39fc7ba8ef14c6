"""Pins of the oracle's draft-input functions (Eq. 1 and the draft layer's norm / QKV / rotary
step) against independent implementations: numpy's matmul on the concatenated input, the Qwen2
modules of the transformers package run in float64, and invariants of the rotary embedding."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl

SMALL = wl.Config("hsr-small", "f32", 4, 2, 16, 3, (((wl.TEXT, 40),),) * 3, 16, 4, False, 96, 200)


def test_hsr_fc_is_linear_on_concatenation():
    c = wl.hsr_case(SMALL, seed=1, rows=5)
    z = oracle.hsr_fc(c.embed, c.token_ids, c.h_prev, c.w_fc, c.b_fc)
    x = np.concatenate([c.embed[c.token_ids], c.h_prev], axis=1).astype(np.float64)
    ref = x @ c.w_fc.astype(np.float64).T + c.b_fc.astype(np.float64)
    np.testing.assert_allclose(z, ref, rtol=1e-12, atol=1e-12)
    lin = torch.nn.Linear(2 * SMALL.hidden, SMALL.hidden, dtype=torch.float64)
    with torch.no_grad():
        lin.weight.copy_(torch.from_numpy(c.w_fc.astype(np.float64)))
        lin.bias.copy_(torch.from_numpy(c.b_fc.astype(np.float64)))
        ref2 = lin(torch.from_numpy(x)).numpy()
    np.testing.assert_allclose(z, ref2, rtol=1e-12, atol=1e-12)


def test_hsr_fc_halves_and_bias():
    """The first H columns of W see the embedding only, the last H the hidden state only, the
    bias is added once: a swapped or dropped half fails here."""
    c = wl.hsr_case(SMALL, seed=2, rows=4)
    H = SMALL.hidden
    z = oracle.hsr_fc(c.embed, c.token_ids, c.h_prev, c.w_fc, c.b_fc)
    z_e = oracle.hsr_fc(c.embed, c.token_ids, np.zeros_like(c.h_prev), c.w_fc, None)
    z_h = oracle.hsr_fc(np.zeros_like(c.embed), c.token_ids, c.h_prev, c.w_fc, None)
    np.testing.assert_allclose(z, z_e + z_h + c.b_fc.astype(np.float64), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(z_e, c.embed[c.token_ids].astype(np.float64) @ c.w_fc[:, :H].astype(np.float64).T,
                               rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(z_h, c.h_prev.astype(np.float64) @ c.w_fc[:, H:].astype(np.float64).T,
                               rtol=1e-12, atol=1e-12)
    # identity projection of the hidden half returns the hidden state, whatever the token is
    W = np.zeros((H, 2 * H), dtype=np.float32)
    W[:, H:] = np.eye(H, dtype=np.float32)
    np.testing.assert_array_equal(oracle.hsr_fc(c.embed, c.token_ids, c.h_prev, W, None),
                                  c.h_prev.astype(np.float64))
    # and of the embedding half the embedding row of that very token id
    W = np.zeros((H, 2 * H), dtype=np.float32)
    W[:, :H] = np.eye(H, dtype=np.float32)
    np.testing.assert_array_equal(oracle.hsr_fc(c.embed, c.token_ids, c.h_prev, W, None),
                                  c.embed[c.token_ids].astype(np.float64))


def test_rope_table_matches_generator_and_transformers():
    pos = np.array([0, 1, 17, 4095, 26111], dtype=np.int32)
    cs, sn = oracle.rope_table(pos, 128, 1.0e6)
    gcs, gsn = wl.rope_rows(pos, 128, 1.0e6)
    np.testing.assert_allclose(cs, gcs, rtol=0, atol=1e-7)
    np.testing.assert_allclose(sn, gsn, rtol=0, atol=1e-7)
    assert cs[0].tolist() == [1.0] * 64 and sn[0].tolist() == [0.0] * 64
    np.testing.assert_allclose(cs[1, 0], np.cos(1.0), atol=1e-15)       # i = 0: frequency 1
    np.testing.assert_allclose(sn[2, 0], np.sin(17.0), atol=1e-15)
    np.testing.assert_allclose(cs[2, 32], np.cos(17.0 * 1.0e6 ** -0.5), atol=1e-15)   # i = d/4
    tr = pytest.importorskip("transformers")
    from transformers.models.qwen2.configuration_qwen2 import Qwen2Config
    from transformers.models.qwen2.modeling_qwen2 import Qwen2RotaryEmbedding
    cfg = Qwen2Config(hidden_size=128 * 4, num_attention_heads=4, num_key_value_heads=2,
                      rope_theta=1.0e6, max_position_embeddings=32768)
    rot = Qwen2RotaryEmbedding(cfg)
    tcos, tsin = rot(torch.zeros(1, 1, dtype=torch.float32), torch.from_numpy(pos.astype(np.int64))[None])
    # float32 angles at position 26111 carry ~1e-3 of error: compare the small positions only
    np.testing.assert_allclose(tcos[0, :3, :64].double().numpy(), cs[:3], atol=2e-6)
    np.testing.assert_allclose(tsin[0, :3, 64:].double().numpy(), sn[:3], atol=2e-6)


def test_draft_qkv_against_transformers_modules():
    """RMSNorm, biased projection and rotate-half rotary embedding of the Qwen2 implementation
    in the transformers package.  Its norm casts to float32 internally, hence 1e-6; eps = 0.5
    makes the place of eps in the formula visible at that tolerance."""
    pytest.importorskip("transformers")
    from transformers.models.qwen2.modeling_qwen2 import Qwen2RMSNorm, apply_rotary_pos_emb
    c = wl.hsr_case(SMALL, seed=3, rows=6, positions=np.array([0, 1, 5, 39, 1000, 26111]))
    Hq, Hkv, d, H = SMALL.n_q_heads, SMALL.n_kv_heads, SMALL.head_dim, SMALL.hidden
    rng = np.random.default_rng(5)
    z = rng.standard_normal((6, H)) * 3.0
    q, k, v = oracle.draft_qkv(z, c.norm_weight, 0.5, c.w_qkv, c.b_qkv, c.rope_cos, c.rope_sin,
                               Hq, Hkv, d)
    norm = Qwen2RMSNorm(H, eps=0.5).double()
    with torch.no_grad():
        norm.weight.copy_(torch.from_numpy(c.norm_weight.astype(np.float64)))
        u = norm(torch.from_numpy(z))
        y = u @ torch.from_numpy(c.w_qkv.astype(np.float64)).T + torch.from_numpy(c.b_qkv.astype(np.float64))
        tq = y[:, :Hq * d].reshape(6, Hq, d).transpose(0, 1)[None]          # [1, heads, M, d]
        tk = y[:, Hq * d:(Hq + Hkv) * d].reshape(6, Hkv, d).transpose(0, 1)[None]
        tv = y[:, (Hq + Hkv) * d:].reshape(6, Hkv, d)
        cos = torch.from_numpy(np.concatenate([c.rope_cos, c.rope_cos], axis=1).astype(np.float64))[None]
        sin = torch.from_numpy(np.concatenate([c.rope_sin, c.rope_sin], axis=1).astype(np.float64))[None]
        rq, rk = apply_rotary_pos_emb(tq, tk, cos, sin)
    np.testing.assert_allclose(q, rq[0].transpose(0, 1).numpy(), rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(k, rk[0].transpose(0, 1).numpy(), rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(v, tv.numpy(), rtol=1e-6, atol=1e-6)


def test_draft_qkv_invariants():
    c = wl.hsr_case(SMALL, seed=4, rows=4, positions=np.array([3, 3, 10, 12]))
    Hq, Hkv, d, H = SMALL.n_q_heads, SMALL.n_kv_heads, SMALL.head_dim, SMALL.hidden
    rng = np.random.default_rng(6)
    z = rng.standard_normal((4, H))
    z[1] = 7.5 * z[0]                       # RMSNorm removes a positive row scale
    args = (c.norm_weight, 0.0, c.w_qkv, c.b_qkv)
    q, k, v = oracle.draft_qkv(z, *args, c.rope_cos, c.rope_sin, Hq, Hkv, d)
    np.testing.assert_allclose(q[1], q[0], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(v[1], v[0], rtol=1e-12, atol=1e-12)
    # position 0 (cos = 1, sin = 0) leaves q and k unrotated: the plain projection
    one, zero = np.ones_like(c.rope_cos), np.zeros_like(c.rope_sin)
    q0, k0, v0 = oracle.draft_qkv(z, *args, one, zero, Hq, Hkv, d)
    u = z / np.sqrt((z * z).mean(axis=1, keepdims=True)) * c.norm_weight.astype(np.float64)
    y = u @ c.w_qkv.astype(np.float64).T + c.b_qkv.astype(np.float64)
    np.testing.assert_allclose(q0.reshape(4, -1), y[:, :Hq * d], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(k0.reshape(4, -1), y[:, Hq * d:(Hq + Hkv) * d], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(v0.reshape(4, -1), y[:, (Hq + Hkv) * d:], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(v, v0, rtol=0, atol=0)          # values are never rotated
    # a rotation: norms of every (i, i + d/2) pair are kept ...
    half = d // 2
    # (the case's float32 table is a rotation to 1e-7 only)
    np.testing.assert_allclose(q[..., :half] ** 2 + q[..., half:] ** 2,
                               q0[..., :half] ** 2 + q0[..., half:] ** 2, rtol=1e-6, atol=1e-7)
    # ... and q.k depends on the position difference only: shift both positions by 1000
    pos = np.array([3, 3, 10, 12])
    cs2, sn2 = oracle.rope_table(pos + 1000, d)
    cs1, sn1 = oracle.rope_table(pos, d)
    qa, ka, _ = oracle.draft_qkv(z, *args, cs1, sn1, Hq, Hkv, d)
    np.testing.assert_allclose(ka[..., :half] ** 2 + ka[..., half:] ** 2,
                               k0[..., :half] ** 2 + k0[..., half:] ** 2, rtol=1e-11, atol=1e-12)
    qb, kb, _ = oracle.draft_qkv(z, *args, cs2, sn2, Hq, Hkv, d)
    dots_a = np.einsum("mhd,ncd->mnhc", qa, ka)
    dots_b = np.einsum("mhd,ncd->mnhc", qb, kb)
    np.testing.assert_allclose(dots_a, dots_b, rtol=1e-9, atol=1e-9)
    # sign convention: rotating e_0 (pair (0, d/2)) by +90 degrees gives +e_{d/2}
    W = np.zeros_like(c.w_qkv)
    W[0, 0] = 1.0                            # q head 0 feature 0 reads z[0]
    g = np.ones(H)
    zz = np.zeros((1, H)); zz[0, 0] = 2.0
    cs = np.zeros((1, half)); sn = np.ones((1, half))
    qq, _, _ = oracle.draft_qkv(zz, g, 0.0, W, None, cs, sn, Hq, Hkv, d)
    val = 2.0 / np.sqrt(4.0 / H)
    np.testing.assert_allclose(qq[0, 0, half], val, rtol=1e-12)
    np.testing.assert_allclose(qq[0, 0, 0], 0.0, atol=1e-12)
