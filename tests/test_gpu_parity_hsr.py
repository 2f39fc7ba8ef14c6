"""GPU parity of the draft's input side (sparrow_hsr_fc, sparrow_draft_qkv_append) against the CPU
fp64 oracle, element by element on the same seeded inputs.

Tolerances.  Inputs are exact in the storage type and products accumulate in fp32, so an fp32
result differs from fp64 by ~K * 2^-24 relative to the sum of |terms| (K <= 8192: 1e-4 of the
output scale is a safe bound).  A bf16 result is rounded once on output (2^-9 relative); the QKV
step also rounds the normalised activations to bf16 on their way into the matrix cores (2^-9 per
element, random signs: ~2^-9 of the output scale after the dot product).  Both fit the 2e-2
(absolute, on outputs of order 1, plus 2e-2 relative) used for the bf16 attention outputs."""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu
TOL = {"f32": (1e-4, 1e-4), "bf16": (2e-2, 2e-2)}     # (atol, rtol)


@pytest.fixture(scope="module")
def sp():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2602_15318_amd as sp_
    return sp_


from gpu_util import dev, host  # noqa: E402


def _cfg(dtype, Hq, Hkv, d, H):
    return wl.Config(f"hsr-{dtype}-{H}", dtype, Hq, Hkv, d, 1, (((wl.TEXT, 64),),), 32, 4, False, H, 2048)


def _close(got, ref, dtype, what):
    atol, rtol = TOL[dtype]
    excess = np.abs(got - ref) - (atol + rtol * np.abs(ref))
    assert excess.max() <= 0, f"{what}: max |err| {np.abs(got - ref).max():.3e}, over the bound by {excess.max():.3e}"


SHAPES = [
    ("f32", 4, 1, 64, 256),        # plain-ALU kernels, the tiny fp32 configuration's widths
    ("bf16", 4, 2, 64, 512),       # plain-ALU kernels in bf16
    ("bf16", 28, 4, 128, 3584),    # matrix-core kernels, Qwen2.5-VL-7B widths (7 slices)
    ("bf16", 32, 8, 128, 4096),    # matrix-core kernels, 8 slices
]


@pytest.mark.parametrize("dtype,Hq,Hkv,d,H", SHAPES)
@pytest.mark.parametrize("M", [1, 9, 16, 17, 64])
def test_hsr_fc(sp, oracle, dtype, Hq, Hkv, d, H, M):
    cfg = _cfg(dtype, Hq, Hkv, d, H)
    c = wl.hsr_case(cfg, seed=M, rows=M, vocab=2048)
    z = sp.hsr_fc(dev(c.embed, dtype), dev(c.token_ids), dev(c.h_prev, dtype), dev(c.w_fc, dtype),
                  dev(c.b_fc, dtype))
    torch.cuda.synchronize()
    ref = oracle.hsr_fc(c.embed, c.token_ids, c.h_prev, c.w_fc, c.b_fc)
    _close(host(z), ref, dtype, f"hsr_fc {dtype} H={H} M={M}")
    if M == 16:       # no bias
        z = sp.hsr_fc(dev(c.embed, dtype), dev(c.token_ids), dev(c.h_prev, dtype), dev(c.w_fc, dtype), None)
        torch.cuda.synchronize()
        _close(host(z), oracle.hsr_fc(c.embed, c.token_ids, c.h_prev, c.w_fc, None), dtype, "hsr_fc, no bias")


@pytest.mark.parametrize("dtype,Hq,Hkv,d,H", SHAPES)
@pytest.mark.parametrize("M", [1, 8, 16, 33, 64])
def test_draft_qkv_append(sp, oracle, dtype, Hq, Hkv, d, H, M):
    cfg = _cfg(dtype, Hq, Hkv, d, H)
    rng = np.random.default_rng(1000 + M)
    T = 300
    kv_rows = rng.choice(T, size=M, replace=False).astype(np.int32)
    positions = rng.integers(0, 26112, size=M)
    c = wl.hsr_case(cfg, seed=M + 1, rows=M, vocab=64, positions=positions)
    z = wl.to_storage(rng.standard_normal((M, H), dtype=np.float32) * 1.5, dtype)
    # cache with padded strides: [T, Hkv + 1, d + 16] storage, the call sees the [T, Hkv, d] corner
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    big_k = torch.full((T, Hkv + 1, d + 16), 7.0, dtype=tdt, device="cuda")
    big_v = torch.full((T, Hkv + 1, d + 16), -3.0, dtype=tdt, device="cuda")
    kc, vc = big_k[:, :Hkv, :d], big_v[:, :Hkv, :d]
    q = sp.draft_qkv_append(dev(z, dtype), dev(c.norm_weight, dtype), c.eps, dev(c.w_qkv, dtype),
                            dev(c.b_qkv, dtype), dev(c.rope_cos), dev(c.rope_sin), kv_rows, Hq, kc, vc)
    torch.cuda.synchronize()
    rq, rk, rv = oracle.draft_qkv(z, c.norm_weight, c.eps, c.w_qkv, c.b_qkv, c.rope_cos, c.rope_sin,
                                  Hq, Hkv, d)
    what = f"draft_qkv {dtype} H={H} M={M}"
    _close(host(q), rq, dtype, what + " q")
    _close(host(kc)[kv_rows], rk, dtype, what + " k")
    _close(host(vc)[kv_rows], rv, dtype, what + " v")
    # nothing but the M appended rows (and only their [Hkv, d] corner) changed
    untouched = np.setdiff1d(np.arange(T), kv_rows)
    assert torch.all(big_k[untouched] == 7.0) and torch.all(big_v[untouched] == -3.0)
    assert torch.all(big_k[:, Hkv] == 7.0) and torch.all(big_k[:, :, d:] == 7.0)
    assert torch.all(big_v[:, Hkv] == -3.0) and torch.all(big_v[:, :, d:] == -3.0)


def test_draft_input_chain_feeds_window_attention(sp, oracle):
    """Eq. 1 -> draft layer input -> Eq. 2 on the device, each stage checked against the oracle on
    the device's own (storage-exact) output of the stage before; then the chained result against
    the oracle's own chain, loosely."""
    cfg = wl.Config("hsr-chain", "bf16", 28, 4, 128, 2,
                    (((wl.TEXT, 40), (wl.VISUAL, 900), (wl.TEXT, 60)),
                     ((wl.VISUAL, 500), (wl.TEXT, 90))), 64, 4, False, 3584, 4096)
    dc = wl.draft_case(cfg, seed=3)
    B = 2
    # the new token of each sequence sits at its last position (a text position, last of text_idx)
    positions = np.array([dc.cu_seqlens[b + 1] - dc.cu_seqlens[b] - 1 for b in range(B)])
    kv_rows = np.array([dc.cu_seqlens[b + 1] - 1 for b in range(B)], dtype=np.int32)
    c = wl.hsr_case(cfg, seed=3, rows=B, vocab=4096, positions=positions)
    dt = "bf16"
    z = sp.hsr_fc(dev(c.embed, dt), dev(c.token_ids), dev(c.h_prev, dt), dev(c.w_fc, dt), dev(c.b_fc, dt))
    kc, vc = dev(dc.k, dt), dev(dc.v, dt)
    q = sp.draft_qkv_append(z, dev(c.norm_weight, dt), c.eps, dev(c.w_qkv, dt), dev(c.b_qkv, dt),
                            dev(c.rope_cos), dev(c.rope_sin), kv_rows, cfg.n_q_heads, kc, vc)
    out, _ = sp.draft_window_attn(q, kc, vc, dc.cu_seqlens, dev(dc.text_idx), dc.cu_text, dc.window)
    torch.cuda.synchronize()
    z_ref = oracle.hsr_fc(c.embed, c.token_ids, c.h_prev, c.w_fc, c.b_fc)
    _close(host(z), z_ref, dt, "chain z")
    rq, rk, rv = oracle.draft_qkv(host(z), c.norm_weight, c.eps, c.w_qkv, c.b_qkv, c.rope_cos,
                                  c.rope_sin, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim)
    _close(host(q), rq, dt, "chain q")
    _close(host(kc)[kv_rows], rk, dt, "chain k")
    _close(host(vc)[kv_rows], rv, dt, "chain v")
    o_ref, _ = oracle.draft_window_attn(host(q), host(kc), host(vc), dc.cu_seqlens, dc.text_idx,
                                        dc.cu_text, dc.window)
    _close(host(out), o_ref, dt, "chain attention on the device's q/k/v")
    # the oracle's own chain, end to end.  The device rounds z, q, k and v to bf16 between the
    # stages (2^-9 relative each), the oracle's chain does not: a score q.k/sqrt(d) of magnitude up
    # to ~6 then moves by up to ~6 * 3 * 2^-9 = 0.035, its softmax weight by 3.5 % of itself, and an
    # output element (a weighted mean of v's of magnitude up to ~1.5) by up to ~0.05, on top of the
    # 2e-2 of the attention itself when every rounding goes one way: 6e-2 bounds the worst case,
    # the stage-by-stage checks above are the tight ones
    k2, v2 = dc.k.astype(np.float64), dc.v.astype(np.float64)
    q2, kk, vv = oracle.draft_qkv(z_ref, c.norm_weight, c.eps, c.w_qkv, c.b_qkv, c.rope_cos,
                                  c.rope_sin, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim)
    k2[kv_rows], v2[kv_rows] = kk, vv
    o2, _ = oracle.draft_window_attn(q2, k2, v2, dc.cu_seqlens, dc.text_idx, dc.cu_text, dc.window)
    assert np.abs(host(out) - o2).max() <= 6e-2


def test_hsr_argument_errors(sp):
    H, M = 256, 2
    f = lambda *s: torch.zeros(*s, device="cuda")     # noqa: E731
    tok = torch.zeros(M, dtype=torch.int32, device="cuda")
    with pytest.raises(sp.SparrowError) as e:
        sp.lib  # noqa: B018
        from paper_2602_15318_amd import binding as b
        b._check(b.lib.sparrow_hsr_fc(0, b._ptr(f(8, H)), b._ptr(tok), b._ptr(f(M, H)), b._ptr(f(H, 2 * H)),
                                      None, 65, H, 8, b._ptr(f(M, H)), None))
    assert e.value.code == -2 and "65" in str(e.value)
    with pytest.raises(sp.SparrowError) as e:
        b._check(b.lib.sparrow_hsr_fc(0, None, b._ptr(tok), b._ptr(f(M, H)), b._ptr(f(H, 2 * H)),
                                      None, M, H, 8, b._ptr(f(M, H)), None))
    assert e.value.code == -1
    kc, vc = f(10, 1, 64), f(10, 1, 64)
    args = (f(M, H), f(H), 1e-6, f(6 * 64, H), None, f(M, 32), f(M, 32))
    with pytest.raises(sp.SparrowError) as e:        # both tokens to the same cache row
        sp.draft_qkv_append(*args, np.array([3, 3]), 4, kc, vc)
    assert e.value.code == -1 and "same cache row" in str(e.value)
    with pytest.raises(sp.SparrowError) as e:
        sp.draft_qkv_append(*args, np.array([-1, 3]), 4, kc, vc)
    assert e.value.code == -1
    # M = 0 is a no-op
    assert b.lib.sparrow_hsr_fc(0, None, None, None, None, None, 0, H, 8, None, None) == 0
