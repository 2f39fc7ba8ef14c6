"""The calls are graph-capturable (no allocation, no synchronisation, no host reads after return):
a captured step replayed several times, with eager work in between, reproduces the eager result
bit for bit.  Also: the profiling hook (partial pass, then combine pass) equals the single call."""
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


from gpu_util import dev  # noqa: E402


def test_graph_replay_matches_eager(sp):
    import torch
    cfg = wl.Config("G", "bf16", 28, 4, 128, 1,
                    (((wl.TEXT, 100), (wl.VISUAL, 3000), (wl.TEXT, 131)),), 128, 8, False, 3584, 8192)
    v = wl.verify_case(cfg, 3)
    d = wl.draft_case(cfg, 3)
    a = wl.accept_case(cfg, 3)
    q, k, vv = dev(v.q, "bf16"), dev(v.k, "bf16"), dev(v.v, "bf16")
    dq, dk, dv, dti = dev(d.q, "bf16"), dev(d.k, "bf16"), dev(d.v, "bf16"), dev(d.text_idx)
    hid, W, ids = dev(a.hidden, "bf16"), dev(a.lm_head, "bf16"), dev(a.draft_ids)
    n_q = cfg.n_q
    ws_v = torch.empty(sp.verify_attn_workspace_bytes(q, k, vv, 1, n_q, int(v.cu_seqlens[-1])),
                       dtype=torch.uint8, device="cuda")
    ws_a = torch.empty(sp.accept_workspace_bytes(1, 1, n_q, cfg.hidden, cfg.vocab), dtype=torch.uint8,
                       device="cuda")

    def make_outputs():
        return (torch.zeros_like(q), torch.zeros_like(dq),
                {"target_ids": torch.zeros(n_q + 1, dtype=torch.int32, device="cuda"),
                 "accept_len": torch.zeros(1, dtype=torch.int32, device="cuda"),
                 "accept_path": torch.zeros(1, n_q, dtype=torch.int32, device="cuda"),
                 "bonus_id": torch.zeros(1, dtype=torch.int32, device="cuda")})

    def step(o_v, o_d, o_a):
        sp.draft_window_attn(dq, dk, dv, d.cu_seqlens, dti, d.cu_text, d.window, out=o_d, want_lse=False)
        sp.verify_attn(q, k, vv, v.cu_seqlens, None, n_q, out=o_v, want_lse=False, workspace=ws_v)
        sp.accept(hid, W, ids, None, 1, n_q, workspace=ws_a, outputs=o_a)

    eager = make_outputs()
    step(*eager)
    torch.cuda.synchronize()
    captured = make_outputs()
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        step(*captured)
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    with torch.cuda.graph(g):
        step(*captured)
    for rep in range(4):
        for t in (captured[0], captured[1], *captured[2].values()):
            t.zero_()                                   # eager work between the replays
        ws_v.random_(0, 255)                            # the workspace carries no state between calls
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(captured[0], eager[0]), f"verify output differs on replay {rep}"
        assert torch.equal(captured[1], eager[1]), f"draft output differs on replay {rep}"
        for key in eager[2]:
            assert torch.equal(captured[2][key], eager[2][key]), f"{key} differs on replay {rep}"


@pytest.mark.parametrize("dtype,Hq,Hkv,d", [("bf16", 28, 4, 128), ("f32", 4, 1, 64)])
def test_partial_then_combine_equals_single_call(sp, dtype, Hq, Hkv, d):
    import torch
    cfg = wl.Config("P", dtype, Hq, Hkv, d, 1, None, 16, 6, False, 64, 128)
    c = wl.verify_case(cfg, 9, layouts=(((wl.TEXT, 1500),), ((wl.TEXT, 333),)), n_q=6, parent=None)
    q, k, v = dev(c.q, dtype), dev(c.k, dtype), dev(c.v, dtype)
    ws = torch.zeros(sp.verify_attn_workspace_bytes(q, k, v, 2, 6, int(c.cu_seqlens[-1])),
                     dtype=torch.uint8, device="cuda")
    ref, ref_lse = sp.verify_attn(q, k, v, c.cu_seqlens, None, 6, workspace=ws)
    out = torch.zeros_like(q)
    lse = torch.zeros_like(ref_lse)
    ws.zero_()
    sp.verify_attn(q, k, v, c.cu_seqlens, None, 6, out=out, lse=lse, workspace=ws, passes=1)
    torch.cuda.synchronize()
    assert not out.any(), "the partial pass must not write the output"
    sp.verify_attn(q, k, v, c.cu_seqlens, None, 6, out=out, lse=lse, workspace=ws, passes=2)
    torch.cuda.synchronize()
    assert torch.equal(out, ref) and torch.equal(lse, ref_lse)
