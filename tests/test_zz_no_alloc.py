"""sparrow_verify_attn_static (the verification attention on the library's own static scratch,
for callers that cannot allocate) against sparrow_verify_attn on the same inputs, through the
C ABI.  The two share their kernels, so the outputs must agree bit for bit (and with them to the
tolerance of the attention parity tests against the oracle); two calls in a row, the second on a
smaller input, so that what the first call left in the scratch is seen not to matter."""
import ctypes

import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sp():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2602_15318_amd as sp_
    return sp_


from gpu_util import check_attn, dev, host  # noqa: E402


def _cfg():
    return wl.Config("S", "bf16", 28, 4, 128, 1, None, 16, 8, False, 64, 128)


def _both(sp, c):
    """(out, lse) of the static entry point called through the raw C symbol, and of
    sparrow_verify_attn."""
    from paper_2602_15318_amd import binding as b
    q, k, v = dev(c.q, "bf16"), dev(c.k, "bf16"), dev(c.v, "bf16")
    par = None if c.parent is None else dev(c.parent)
    ref_out, ref_lse = sp.verify_attn(q, k, v, c.cu_seqlens, par, c.n_q)
    out = torch.full_like(q, float("nan"))
    lse = torch.full(q.shape[:2], float("nan"), dtype=torch.float32, device=q.device)
    desc = b.AttnDesc(b.SPARROW_BF16, q.shape[1], k.shape[1], q.shape[2], 0.0, k.stride(0), k.stride(1), 0)
    cu = np.ascontiguousarray(c.cu_seqlens, dtype=np.int32)
    rc = b.lib.sparrow_verify_attn_static(
        ctypes.byref(desc), b._ptr(q), b._ptr(k), b._ptr(v),
        cu.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), b._ptr(par), len(cu) - 1, c.n_q,
        b._ptr(out), b._ptr(lse), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, sp.last_error()
    torch.cuda.synchronize()
    return (out, lse), (ref_out, ref_lse)


def test_static_scratch_entry_matches_the_workspace_entry(sp, oracle):
    cfg = _cfg()
    big = wl.verify_case(cfg, seed=1, layouts=(((wl.TEXT, 40), (wl.VISUAL, 9000), (wl.TEXT, 60)),
                                               ((wl.VISUAL, 2500), (wl.TEXT, 33))),
                         n_q=len(wl.pruned_tree(2, 30, (4, 3, 2, 2))), parent=wl.pruned_tree(2, 30, (4, 3, 2, 2)))
    small = wl.verify_case(cfg, seed=2, layouts=(((wl.TEXT, 20), (wl.VISUAL, 700), (wl.TEXT, 11)),),
                           n_q=5, parent=None)
    for c, what in ((big, "first call: batch of two, tree of 30 nodes"),
                    (small, "second call: one short sequence, chain of 5")):
        (out, lse), (ref_out, ref_lse) = _both(sp, c)
        assert torch.equal(out.view(torch.int16), ref_out.view(torch.int16)), what
        assert torch.equal(lse, ref_lse), what
        o_ref, l_ref = oracle.verify_attn(c.q, c.k, c.v, c.cu_seqlens, c.parent, c.n_q)
        check_attn(host(out), o_ref, "bf16", what)
        assert np.abs(host(lse) - l_ref).max() <= 4e-3, what


def test_static_scratch_entry_rejects_what_does_not_fit(sp):
    """64 sequences with 64-node trees need ~30 MB of split partials: more than the 16 MiB array."""
    from paper_2602_15318_amd import binding as b
    B, n_q, L = 64, 64, 40
    T = B * (L + n_q)
    q = torch.zeros(B * n_q, 28, 128, dtype=torch.bfloat16, device="cuda")
    k = torch.zeros(T, 4, 128, dtype=torch.bfloat16, device="cuda")
    cu = np.arange(B + 1, dtype=np.int32) * (L + n_q)
    assert sp.verify_attn_workspace_bytes(q, k, k, B, n_q, T) > sp.STATIC_WS_BYTES
    out = torch.zeros_like(q)
    with pytest.raises(sp.SparrowError) as e:
        sp.verify_attn_static(q, k, k, cu, None, n_q, out)
    assert e.value.code == -2 and "static scratch" in str(e.value)
    # and the ordinary validation still comes first
    with pytest.raises(sp.SparrowError) as e:
        sp.verify_attn_static(q, k, k, np.array([0, 3], dtype=np.int32), None, n_q, out)
    assert e.value.code == -1


def test_static_scratch_entry_in_a_captured_graph(sp):
    """The use the entry point is for: captured in a HIP graph (after one call outside capture,
    which looks the scratch address up), replayed several times with eager work in between, each
    replay equal to the eager result bit for bit."""
    cfg = _cfg()
    c = wl.verify_case(cfg, seed=5, layouts=(((wl.TEXT, 30), (wl.VISUAL, 5000), (wl.TEXT, 70)),), n_q=8,
                       parent=None)
    q, k, v = dev(c.q, "bf16"), dev(c.k, "bf16"), dev(c.v, "bf16")
    eager = torch.zeros_like(q)
    sp.verify_attn_static(q, k, v, c.cu_seqlens, None, 8, eager)
    torch.cuda.synchronize()
    out = torch.zeros_like(q)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        sp.verify_attn_static(q, k, v, c.cu_seqlens, None, 8, out)
    other = wl.verify_case(cfg, seed=6, layouts=(((wl.TEXT, 900),),), n_q=3, parent=None)
    oq, ok_, ov = dev(other.q, "bf16"), dev(other.k, "bf16"), dev(other.v, "bf16")
    scratch_user = torch.zeros_like(oq)
    for rep in range(3):
        out.zero_()
        # an eager call on the same scratch between the replays leaves other contents in it
        sp.verify_attn_static(oq, ok_, ov, other.cu_seqlens, None, 3, scratch_user)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), f"replay {rep}"
