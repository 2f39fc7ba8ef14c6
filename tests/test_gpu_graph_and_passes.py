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


def test_graph_replay_of_the_surrounding_steps(sp):
    """Draft input, dynamic tree, acceptance at T = 1 and commit in one captured graph: replays
    with scribbled workspaces and outputs in between reproduce the eager results bit for bit."""
    import torch
    cfg = wl.Config("G2", "bf16", 28, 4, 128, 1,
                    (((wl.TEXT, 60), (wl.VISUAL, 800), (wl.TEXT, 40)),), 64, 6, False, 3584, 4096)
    n_q, H, V = cfg.n_q, cfg.hidden, cfg.vocab
    hc = wl.hsr_case(cfg, 5, rows=1, vocab=V)
    d = wl.draft_case(cfg, 5)
    v = wl.verify_case(cfg, 5)
    a = wl.accept_case(cfg, 5, planted=True)
    bf = "bf16"
    emb, tok, hp = dev(hc.embed, bf), dev(hc.token_ids), dev(hc.h_prev, bf)
    wfc, bfc, g_, wqkv, bqkv = (dev(hc.w_fc, bf), dev(hc.b_fc, bf), dev(hc.norm_weight, bf),
                                dev(hc.w_qkv, bf), dev(hc.b_qkv, bf))
    cs, sn = dev(hc.rope_cos), dev(hc.rope_sin)
    dk, dv = dev(d.k, bf), dev(d.v, bf)
    kv_row = np.array([int(d.cu_seqlens[1]) - 1], dtype=np.int32)
    vk, vv = dev(v.k, bf), dev(v.v, bf)
    hid, W = dev(a.hidden, bf), dev(a.lm_head, bf)
    draft = a.planted_ids[:n_q].copy()
    draft[3] = (draft[3] + 1) % V
    draft = dev(draft)
    ua = torch.full((1, n_q), 0.01, device="cuda")
    ub = torch.full((1,), 0.5, device="cuda")
    ws_s = torch.empty(sp.accept_sample_workspace_bytes(1, 1, n_q, H, V), dtype=torch.uint8, device="cuda")
    ws_t = torch.empty(int(sp.lib.sparrow_draft_topk_workspace(1, n_q + 1, H, V, 4)), dtype=torch.uint8,
                       device="cuda")

    def make():
        return {"z": torch.zeros(1, H, dtype=torch.bfloat16, device="cuda"),
                "q": torch.zeros(1, 28, 128, dtype=torch.bfloat16, device="cuda"),
                "s": {"accept_len": torch.zeros(1, dtype=torch.int32, device="cuda"),
                      "accept_path": torch.zeros(1, n_q, dtype=torch.int32, device="cuda"),
                      "bonus_id": torch.zeros(1, dtype=torch.int32, device="cuda")},
                "next": torch.zeros(1, H, dtype=torch.bfloat16, device="cuda"),
                "k": vk.clone(), "v": vv.clone(), "dk": dk.clone(), "dv": dv.clone()}

    def step(o):
        sp.hsr_fc(emb, tok, hp, wfc, bfc, out=o["z"])
        sp.draft_qkv_append(o["z"], g_, hc.eps, wqkv, bqkv, cs, sn, kv_row, 28, o["dk"], o["dv"], q_out=o["q"])
        ids, lp = sp.draft_topk(hid, W, 4, workspace=ws_t)
        o["ids"], o["lp"] = ids, lp
        sp.accept_sample(hid, W, draft, None, 1, n_q, 1.0, ua, ub, workspace=ws_s, outputs=o["s"])
        sp.kv_commit([o["k"]], [o["v"]], v.cu_seqlens, n_q, o["s"]["accept_path"], o["s"]["accept_len"],
                     hidden_rows=hid, next_hidden=o["next"])

    eager = make()
    step(eager)
    torch.cuda.synchronize()
    assert eager["s"]["accept_len"].item() == 3          # planted, u = 0.01: three drafts accepted
    cap = make()
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        step(cap)
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    with torch.cuda.graph(g):
        step(cap)
    for rep in range(3):
        for t in (cap["z"], cap["q"], cap["next"], cap["ids"], cap["lp"], *cap["s"].values()):
            t.zero_()
        cap["k"].copy_(vk); cap["v"].copy_(vv); cap["dk"].copy_(dk); cap["dv"].copy_(dv)
        ws_s.random_(0, 255); ws_t.random_(0, 255)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for key in ("z", "q", "next", "k", "v", "dk", "dv", "ids", "lp"):
            assert torch.equal(cap[key], eager[key]), f"{key} differs on replay {rep}"
        for key in eager["s"]:
            assert torch.equal(cap["s"][key], eager["s"][key]), f"{key} differs on replay {rep}"


def test_stream_read_runs_and_leaves_its_input_alone(sp):
    """The measurement aid reads a buffer and writes nothing but (at most) its 4-byte sink."""
    import torch
    x = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    keep = x.clone()
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    for n in (4, 1 << 10, (1 << 20) - 4, 1 << 20):        # ragged tails of the unrolled loop
        sp.stream_read(x[:n], sink)
    torch.cuda.synchronize()
    assert torch.equal(x, keep)
    # the loads are live: one 16-byte load whose words XOR to all ones reaches the sink
    w = torch.tensor([-1, 0, 0, 0], dtype=torch.int32, device="cuda")
    sp.stream_read(w, sink)
    torch.cuda.synchronize()
    assert int(sink.item()) == -1


def test_debug_validators_on_device_arrays(sp):
    """The synchronous precondition checks on device-resident arrays."""
    import torch
    par = wl.pruned_tree(0, 30, (4, 3, 2, 2))
    d_par = torch.from_numpy(par).cuda()
    sp.debug_validate_parent(d_par, 30)
    trees = torch.from_numpy(np.stack([wl.pruned_tree(i, 30, (4, 3, 2, 2)) for i in range(4)])).cuda()
    sp.debug_validate_parent(trees, 30, B=4)
    trees[3, 17] = 17
    with pytest.raises(sp.SparrowError) as e:
        sp.debug_validate_parent(trees, 30, B=4)
    assert e.value.code == -1 and "tree 3: parent[17] = 17" in str(e.value)
    c = wl.draft_case(wl.C4, 0)
    tix = torch.from_numpy(c.text_idx).cuda()
    sp.debug_validate_text_idx(tix, c.cu_seqlens, c.cu_text)
    tix[int(c.cu_text[5]) + 1] = 10 ** 6
    with pytest.raises(sp.SparrowError) as e:
        sp.debug_validate_text_idx(tix, c.cu_seqlens, c.cu_text)
    assert e.value.code == -1 and "sequence 5" in str(e.value)


def test_stream_read_shapes_run(sp):
    """The measurement aid (a kernel that only reads a byte range) in every launch shape bench.py
    sweeps: all four numbers of loads in flight, both sweep orders, ragged sizes.  It computes
    nothing that could be compared; the calls must succeed and leave the buffer untouched."""
    import torch
    buf = torch.arange(3 * 1024 * 1024 + 5000, dtype=torch.int32, device="cuda")      # 12.6 MB
    keep = buf.clone()
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    for in_flight in (2, 4, 8, 16):
        for regions in (0, 1):
            for wgs in (1, 256, 2048):
                sp.stream_read(buf, sink, shape=(wgs, in_flight, regions))
    sp.stream_read(buf[:4], sink)                     # 16 bytes: the shortest range
    sp.stream_read(buf, sink)
    torch.cuda.synchronize()
    assert torch.equal(buf, keep)
    with pytest.raises(sp.SparrowError):
        sp.stream_read(buf, sink, shape=(256, 3, 0))
