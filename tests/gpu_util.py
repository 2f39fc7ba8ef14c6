"""Helpers of the GPU parity tests: move seeded workload tensors to the device and call the HIP
library through its C-ABI binding."""
import numpy as np
import torch

import workloads as wl

TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}
# Tolerances on attention outputs (max-abs error; also applied relative to max|reference|).
ATOL = {"f32": 1e-5, "bf16": 2e-2}


def dev(x: np.ndarray, dtype: str = None):
    t = torch.from_numpy(np.ascontiguousarray(x)).to("cuda")
    return t if dtype is None else t.to(TORCH_DTYPE[dtype])


def host(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy() if t.is_floating_point() else t.cpu().numpy()


def run_draft(sp, c: wl.DraftCase, **kw):
    dt = c.cfg.dtype
    out, lse = sp.draft_window_attn(dev(c.q, dt), dev(c.k, dt), dev(c.v, dt), c.cu_seqlens,
                                    dev(c.text_idx), c.cu_text, c.window, **kw)
    torch.cuda.synchronize()
    return host(out), host(lse)


def run_verify(sp, c: wl.VerifyCase, **kw):
    dt = c.cfg.dtype
    par = None if c.parent is None else dev(c.parent)
    out, lse = sp.verify_attn(dev(c.q, dt), dev(c.k, dt), dev(c.v, dt), c.cu_seqlens, par, c.n_q,
                              **kw)
    torch.cuda.synchronize()
    return host(out), host(lse)


def run_accept(sp, c: wl.AcceptCase, B: int, draft_ids=None, lm_head_dev=None):
    dt = c.cfg.dtype
    par = None if c.parent is None else dev(c.parent)
    W = lm_head_dev if lm_head_dev is not None else dev(c.lm_head, dt)
    ids = c.draft_ids if draft_ids is None else draft_ids
    r = sp.accept(dev(c.hidden, dt), W, dev(np.asarray(ids, dtype=np.int32)), par, B, c.n_q)
    torch.cuda.synchronize()
    return {k: host(v) for k, v in r.items()}


def check_attn(out, ref, dtype: str, what: str = ""):
    """max-abs error within the stated tolerance, both absolutely and relative to the largest
    reference magnitude (the absolute bound alone is vacuous when outputs are ~0.01)."""
    assert out.shape == ref.shape
    assert np.isfinite(out).all(), f"{what}: non-finite output"
    err = float(np.abs(out - ref).max())
    scale = float(np.abs(ref).max())
    tol = ATOL[dtype]
    assert err <= tol, f"{what}: max-abs error {err:.3e} > {tol}"
    assert err <= tol * max(scale, 1e-30), f"{what}: error {err:.3e} vs max|ref| {scale:.3e}: relative {err/scale:.3e} > {tol}"
    return err, scale
