"""GPU parity of sparrow_kv_commit against the CPU oracle: pure data movement, so every cache row
of every layer and the gathered hidden rows must match bit for bit."""
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


from gpu_util import dev, host, run_accept  # noqa: E402


def _random_paths(rng, parent, B, n_q, lens):
    """Root-to-node paths of the given lengths (or as deep as the tree allows), -1 padded."""
    par = wl.chain_parent(n_q) if parent is None else parent
    path = np.full((B, n_q), -1, dtype=np.int32)
    alen = np.zeros(B, dtype=np.int32)
    for b in range(B):
        cur = -1
        for j in range(lens[b]):
            kids = np.flatnonzero(par == cur)
            if len(kids) == 0:
                break
            cur = int(rng.choice(kids))
            path[b, j] = cur
            alen[b] = j + 1
    return path, alen


@pytest.mark.parametrize("dtype,Hkv,d,n_q,tree,B,n_layers", [
    ("bf16", 4, 128, 8, False, 1, 3),
    ("bf16", 4, 128, 60, True, 2, 2),
    ("bf16", 2, 64, 12, True, 3, 1),
    ("f32", 1, 64, 4, False, 2, 2),
    ("f32", 2, 128, 64, False, 1, 1),       # the longest chain, 512-byte rows: all 8 passes
])
def test_kv_commit_bit_exact(sp, oracle, dtype, Hkv, d, n_q, tree, B, n_layers):
    rng = np.random.default_rng(n_q * 7 + B)
    parent = wl.pruned_tree(5, n_q, (4, 3, 2, 2, 1, 1)) if tree else None
    if tree:
        assert len(parent) == n_q
    ctx = rng.integers(0, 40, size=B)
    cu = np.concatenate(([0], np.cumsum(ctx + n_q))).astype(np.int32)
    lens = [int(rng.integers(0, n_q + 1)) for _ in range(B)]
    if B > 1:
        lens[0] = 0                        # one sequence accepts nothing
    path, alen = _random_paths(rng, parent, B, n_q, lens)
    T, H = int(cu[-1]), 256
    ks = [wl.to_storage(rng.standard_normal((T, Hkv, d), dtype=np.float32), dtype) for _ in range(n_layers)]
    vs = [wl.to_storage(rng.standard_normal((T, Hkv, d), dtype=np.float32), dtype) for _ in range(n_layers)]
    hid = wl.to_storage(rng.standard_normal((B * (n_q + 1), H), dtype=np.float32), dtype)
    dk, dv = [dev(x, dtype) for x in ks], [dev(x, dtype) for x in vs]
    nh = sp.kv_commit(dk, dv, cu, n_q, dev(path), dev(alen), hidden_rows=dev(hid, dtype))
    torch.cuda.synchronize()
    for l in range(n_layers):
        np.testing.assert_array_equal(host(dk[l]), oracle.kv_commit(ks[l], cu, n_q, path, alen),
                                      err_msg=f"layer {l} K")
        np.testing.assert_array_equal(host(dv[l]), oracle.kv_commit(vs[l], cu, n_q, path, alen),
                                      err_msg=f"layer {l} V")
    np.testing.assert_array_equal(host(nh), oracle.next_hidden(hid, B, n_q, path, alen))


def test_accept_then_commit_on_device(sp, oracle):
    """sparrow_accept's device outputs go straight into sparrow_kv_commit (no host round trip)."""
    cfg = wl.Config("commit-chain", "bf16", 28, 4, 128, 2,
                    (((wl.TEXT, 30), (wl.VISUAL, 200), (wl.TEXT, 26)), ((wl.VISUAL, 90), (wl.TEXT, 21))),
                    32, 6, False, 512, 4096)
    ac = wl.accept_case(cfg, seed=11, planted=True)
    B, n_q = 2, cfg.n_q
    # make sequence 0 accept 4 drafts and sequence 1 accept 2: copy the planted targets
    t = ac.planted_ids.reshape(B, n_q + 1)
    draft = ac.draft_ids.reshape(B, n_q).copy()
    draft[0, :4] = t[0, :4]
    draft[0, 4] = (t[0, 4] + 1) % cfg.vocab
    draft[1, :2] = t[1, :2]
    draft[1, 2] = (t[1, 2] + 1) % cfg.vocab
    ref = oracle.accept_step(ac.hidden, ac.lm_head, draft.reshape(-1), None, B, n_q)
    assert ref["accept_len"].tolist() == [4, 2] and ref["margin"].min() > 1e-3
    vc = wl.verify_case(cfg, seed=11)
    dk, dv = dev(vc.k, "bf16"), dev(vc.v, "bf16")
    hidden = dev(ac.hidden, "bf16")
    res = sp.accept(hidden, dev(ac.lm_head, "bf16"), dev(draft.reshape(-1)), None, B, n_q)
    nh = sp.kv_commit([dk], [dv], vc.cu_seqlens, n_q, res["accept_path"], res["accept_len"],
                      hidden_rows=hidden)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(dk), oracle.kv_commit(vc.k, vc.cu_seqlens, n_q, ref["accept_path"], ref["accept_len"]))
    np.testing.assert_array_equal(host(nh), oracle.next_hidden(ac.hidden, B, n_q, ref["accept_path"], ref["accept_len"]))


def test_kv_commit_argument_errors(sp):
    k = torch.zeros(20, 2, 64, device="cuda")
    path = torch.zeros(1, 4, dtype=torch.int32, device="cuda")
    alen = torch.zeros(1, dtype=torch.int32, device="cuda")
    with pytest.raises(sp.SparrowError) as e:          # sequence shorter than its draft rows
        sp.kv_commit([k], [k.clone()], np.array([0, 3]), 4, path, alen)
    assert e.value.code == -1
    with pytest.raises(sp.SparrowError) as e:
        sp.kv_commit([k] * 65, [k] * 65, np.array([0, 20]), 4, path, alen)
    assert e.value.code == -2 and "65" in str(e.value)
