"""ctypes front end of the CPU fp64 oracle (oracle/sparrow_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The HIP library and its Python binding never
import this package, and this package never imports them.

Every function takes numpy arrays of any float type, widens them to float64
(exact for fp32 / bf16-representable inputs) and returns float64 / int32
arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sparrow_oracle.c")
_LIB = os.path.join(_HERE, "libsparrow_oracle.so")

_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int32)


# SPARROW_ORACLE_SANITIZE=1 (set by tests/test_oracle_sanitized.py for a child process that has the
# AddressSanitizer runtime preloaded): a second library built with -fsanitize=address,undefined,
# so that an out-of-bounds access or undefined behaviour in the oracle aborts the run.
_SANITIZE = os.environ.get("SPARROW_ORACLE_SANITIZE") == "1"
if _SANITIZE:
    _LIB = os.path.join(_HERE, "libsparrow_oracle_san.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
               "-fno-omit-frame-pointer"] if _SANITIZE else ["-O2"]
        cmd = ["gcc", *opt, "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_draft_window_attn.restype = ctypes.c_int
        _lib.oracle_verify_attn.restype = ctypes.c_int
        _lib.oracle_accept.restype = ctypes.c_int
        _lib.oracle_logits.restype = None
        _lib.oracle_argmax.restype = None
        _lib.oracle_hsr_fc.restype = None
        _lib.oracle_draft_qkv.restype = None
        _lib.oracle_rope_table.restype = None
        _lib.oracle_kv_commit.restype = None
        _lib.oracle_accept_sample.restype = ctypes.c_int
        _lib.oracle_accept_sample_q.restype = ctypes.c_int
        _lib.oracle_philox4x32_10.restype = None
        _lib.oracle_philox_uniforms.restype = None
        _lib.oracle_topk_logprob.restype = None
        _lib.oracle_tree_expand.restype = ctypes.c_int
        _lib.oracle_tree_select.restype = ctypes.c_int
        _lib.oracle_next_hidden.restype = None
    return _lib


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a: Optional[np.ndarray], t):
    return None if a is None else a.ctypes.data_as(t)


def default_scale(head_dim: int) -> float:
    """1/sqrt(d) with d the per-head dimension (reading of "d" in Eq. 2)."""
    return 1.0 / float(np.sqrt(float(head_dim)))


def draft_window_attn(q, k, v, cu_seqlens, text_idx, cu_text, window: int,
                      scale: Optional[float] = None) -> Tuple[np.ndarray, np.ndarray]:
    """q [B,Hq,d]; k,v [T,Hkv,d] (position-indexed); returns (out [B,Hq,d], lse [B,Hq])."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, Hq, d = q.shape
    T, Hkv, d2 = k.shape
    assert d2 == d and v.shape == k.shape
    cu, ti, ct = _i32(cu_seqlens), _i32(text_idx), _i32(cu_text)
    assert cu.shape == (B + 1,) and ct.shape == (B + 1,)
    out = np.empty((B, Hq, d), dtype=np.float64)
    lse = np.empty((B, Hq), dtype=np.float64)
    sc = default_scale(d) if scale is None else float(scale)
    rc = _load().oracle_draft_window_attn(
        _ptr(q, _dp), _ptr(k, _dp), _ptr(v, _dp), _ptr(cu, _ip), _ptr(ti, _ip), _ptr(ct, _ip),
        ctypes.c_int(B), ctypes.c_int(Hq), ctypes.c_int(Hkv), ctypes.c_int(d),
        ctypes.c_double(sc), ctypes.c_int(int(window)),
        ctypes.c_int64(Hkv * d), ctypes.c_int64(d), _ptr(out, _dp), _ptr(lse, _dp))
    if rc != 0:
        raise ValueError("oracle_draft_window_attn: invalid arguments")
    return out, lse


def verify_attn(q, k, v, cu_seqlens, parent, n_q: int,
                scale: Optional[float] = None) -> Tuple[np.ndarray, np.ndarray]:
    """q [B*n_q,Hq,d]; k,v [sum(L_b+n_q),Hkv,d]; parent int32 [n_q] or None (chain).
    Returns (out [B*n_q,Hq,d], lse [B*n_q,Hq])."""
    cu = _i32(cu_seqlens)
    B = cu.shape[0] - 1
    if parent is not None and np.ndim(parent) == 2:
        # one tree per sequence [B, n_q]: by definition the per-sequence results, each sequence
        # verified on its own with its own tree
        par2 = _i32(parent)
        assert par2.shape == (B, n_q)
        outs, lses = [], []
        for b in range(B):
            o, l = verify_attn(np.asarray(q)[b * n_q:(b + 1) * n_q], np.asarray(k)[cu[b]:cu[b + 1]],
                               np.asarray(v)[cu[b]:cu[b + 1]], [0, cu[b + 1] - cu[b]], par2[b], n_q, scale)
            outs.append(o)
            lses.append(l)
        return np.concatenate(outs), np.concatenate(lses)
    q, k, v = _f64(q), _f64(k), _f64(v)
    rows, Hq, d = q.shape
    T, Hkv, _ = k.shape
    assert rows == B * n_q and v.shape == k.shape
    par = None if parent is None else _i32(parent)
    out = np.empty((rows, Hq, d), dtype=np.float64)
    lse = np.empty((rows, Hq), dtype=np.float64)
    sc = default_scale(d) if scale is None else float(scale)
    rc = _load().oracle_verify_attn(
        _ptr(q, _dp), _ptr(k, _dp), _ptr(v, _dp), _ptr(cu, _ip), _ptr(par, _ip),
        ctypes.c_int(B), ctypes.c_int(int(n_q)), ctypes.c_int(Hq), ctypes.c_int(Hkv),
        ctypes.c_int(d), ctypes.c_double(sc), ctypes.c_int64(Hkv * d), ctypes.c_int64(d),
        _ptr(out, _dp), _ptr(lse, _dp))
    if rc != 0:
        raise ValueError("oracle_verify_attn: invalid arguments")
    return out, lse


def logits(hidden, lm_head, chunk: int = 8192) -> np.ndarray:
    """hidden [rows,H] x lm_head [V,H]^T -> [rows,V] float64.  The weight matrix
    is widened to float64 a block of rows at a time to bound memory."""
    hidden = _f64(hidden)
    rows, H = hidden.shape
    V = lm_head.shape[0]
    out = np.empty((rows, V), dtype=np.float64)
    lib = _load()
    for v0 in range(0, V, chunk):
        v1 = min(V, v0 + chunk)
        w = _f64(lm_head[v0:v1])
        part = np.empty((rows, v1 - v0), dtype=np.float64)
        lib.oracle_logits(_ptr(hidden, _dp), _ptr(w, _dp), ctypes.c_int(rows), ctypes.c_int(H),
                          ctypes.c_int64(v1 - v0), _ptr(part, _dp))
        out[:, v0:v1] = part
    return out


def argmax(lg) -> Tuple[np.ndarray, np.ndarray]:
    """Per-row greedy token (lowest index on ties) and top-1 minus top-2 margin."""
    lg = _f64(lg)
    rows, V = lg.shape
    ids = np.empty(rows, dtype=np.int32)
    margin = np.empty(rows, dtype=np.float64)
    _load().oracle_argmax(_ptr(lg, _dp), ctypes.c_int(rows), ctypes.c_int64(V),
                          _ptr(ids, _ip), _ptr(margin, _dp))
    return ids, margin


def accept(target_ids, draft_ids, parent, B: int, n_q: int):
    """Returns (accept_len [B], accept_path [B,n_q], bonus_id [B])."""
    t, dr = _i32(target_ids), _i32(draft_ids)
    assert t.shape == (B * (n_q + 1),) and dr.shape == (B * n_q,)
    if parent is not None and np.ndim(parent) == 2:      # one tree per sequence: per-sequence walks
        par2 = _i32(parent)
        assert par2.shape == (B, n_q)
        parts = [accept(t[b * (n_q + 1):(b + 1) * (n_q + 1)], dr[b * n_q:(b + 1) * n_q], par2[b], 1, n_q)
                 for b in range(B)]
        return tuple(np.concatenate([p[i] for p in parts]) for i in range(3))
    par = None if parent is None else _i32(parent)
    alen = np.empty(B, dtype=np.int32)
    path = np.empty((B, max(n_q, 0)), dtype=np.int32)
    bonus = np.empty(B, dtype=np.int32)
    rc = _load().oracle_accept(_ptr(t, _ip), _ptr(dr, _ip), _ptr(par, _ip), ctypes.c_int(B),
                               ctypes.c_int(n_q), _ptr(alen, _ip), _ptr(path, _ip),
                               _ptr(bonus, _ip))
    if rc != 0:
        raise ValueError("oracle_accept: invalid parent array")
    return alen, path, bonus


def accept_step(hidden, lm_head, draft_ids, parent, B: int, n_q: int):
    """lm_head GEMM -> argmax -> greedy acceptance.  Returns a dict with
    target_ids, margin, accept_len, accept_path, bonus_id."""
    lg = logits(hidden, lm_head)
    ids, margin = argmax(lg)
    alen, path, bonus = accept(ids, draft_ids, parent, B, n_q)
    return {"target_ids": ids, "margin": margin, "accept_len": alen,
            "accept_path": path, "bonus_id": bonus}


def hsr_fc(embed, token_ids, h_prev, w_fc, b_fc=None) -> np.ndarray:
    """z = FC(e (+) h) (Eq. 1): embed [vocab, H] (only the rows of token_ids are widened),
    h_prev [M, H], w_fc [H, 2H], b_fc [H] or None.  Returns z [M, H] float64."""
    lib = _load()
    tok = _i32(token_ids)
    e = _f64(np.asarray(embed)[tok])
    h = _f64(h_prev)
    M, H = h.shape
    W = _f64(w_fc)
    assert e.shape == (M, H) and W.shape == (H, 2 * H)
    b = None if b_fc is None else _f64(b_fc)
    z = np.empty((M, H), dtype=np.float64)
    lib.oracle_hsr_fc(_ptr(e, _dp), _ptr(h, _dp), _ptr(W, _dp), _ptr(b, _dp), ctypes.c_int(M),
                      ctypes.c_int(H), _ptr(z, _dp))
    return z


def draft_qkv(z, gamma, eps: float, w_qkv, b_qkv, rope_cos, rope_sin, n_q_heads: int,
              n_kv_heads: int, head_dim: int):
    """RMSNorm -> QKV projection (+ bias) -> rotary embedding of q and k.
    Returns q [M, Hq, d], k [M, Hkv, d], v [M, Hkv, d] float64."""
    lib = _load()
    z = _f64(z)
    M, H = z.shape
    N = (n_q_heads + 2 * n_kv_heads) * head_dim
    W = _f64(w_qkv)
    assert W.shape == (N, H)
    g = _f64(gamma)
    b = None if b_qkv is None else _f64(b_qkv)
    cs, sn = _f64(rope_cos), _f64(rope_sin)
    assert cs.shape == (M, head_dim // 2) and sn.shape == cs.shape
    q = np.empty((M, n_q_heads, head_dim), dtype=np.float64)
    k = np.empty((M, n_kv_heads, head_dim), dtype=np.float64)
    v = np.empty((M, n_kv_heads, head_dim), dtype=np.float64)
    lib.oracle_draft_qkv(_ptr(z, _dp), _ptr(g, _dp), ctypes.c_double(eps), _ptr(W, _dp),
                         _ptr(b, _dp), _ptr(cs, _dp), _ptr(sn, _dp), ctypes.c_int(M),
                         ctypes.c_int(H), ctypes.c_int(n_q_heads), ctypes.c_int(n_kv_heads),
                         ctypes.c_int(head_dim), _ptr(q, _dp), _ptr(k, _dp), _ptr(v, _dp))
    return q, k, v


def rope_table(positions, head_dim: int, theta: float = 1.0e6):
    """(cos, sin) [M, d/2] float64 of the rotate-half rotary embedding."""
    lib = _load()
    pos = _i32(positions)
    M = pos.shape[0]
    cs = np.empty((M, head_dim // 2), dtype=np.float64)
    sn = np.empty_like(cs)
    lib.oracle_rope_table(_ptr(pos, _ip), ctypes.c_int(M), ctypes.c_int(head_dim),
                          ctypes.c_double(theta), _ptr(cs, _dp), _ptr(sn, _dp))
    return cs, sn


def kv_commit(cache, cu_seqlens, n_q: int, accept_path, accept_len) -> np.ndarray:
    """One layer's K or V cache [T, ...] after the accepted draft rows have been moved up behind
    the context, in path order.  Returns a new float64 array of the same shape."""
    lib = _load()
    c = np.array(cache, dtype=np.float64, order="C", copy=True)
    cu = _i32(cu_seqlens)
    B = cu.shape[0] - 1
    path, alen = _i32(accept_path).reshape(B, max(n_q, 0)), _i32(accept_len)
    row_elems = int(np.prod(c.shape[1:]))
    lib.oracle_kv_commit(_ptr(c, _dp), ctypes.c_int64(row_elems), _ptr(cu, _ip), ctypes.c_int(B),
                         ctypes.c_int(n_q), _ptr(path, _ip), _ptr(alen, _ip))
    return c


def next_hidden(hidden, B: int, n_q: int, accept_path, accept_len) -> np.ndarray:
    """[B, H] hidden rows of the last accepted nodes (row 0 of a sequence if none)."""
    lib = _load()
    h = _f64(hidden)
    H = h.shape[1]
    path, alen = _i32(accept_path).reshape(B, max(n_q, 0)), _i32(accept_len)
    out = np.empty((B, H), dtype=np.float64)
    lib.oracle_next_hidden(_ptr(h, _dp), ctypes.c_int(B), ctypes.c_int(n_q), ctypes.c_int(H),
                           _ptr(path, _ip), _ptr(alen, _ip), _ptr(out, _dp))
    return out


def accept_sample(lg, draft_ids, parent, B: int, n_q: int, temperature: float, u_accept, u_bonus):
    """Stochastic (temperature > 0) acceptance on given logits [B*(n_q+1), V].  Returns
    (accept_len [B], accept_path [B, n_q], bonus_id [B], margin [B])."""
    lib = _load()
    lg = _f64(lg)
    V = lg.shape[1]
    assert lg.shape[0] == B * (n_q + 1)
    dr = _i32(draft_ids)
    if parent is not None and np.ndim(parent) == 2:      # one tree per sequence: per-sequence walks
        par2 = _i32(parent)
        assert par2.shape == (B, n_q)
        ua2, ub2 = np.asarray(u_accept).reshape(B, n_q), np.asarray(u_bonus).reshape(B)
        parts = [accept_sample(lg[b * (n_q + 1):(b + 1) * (n_q + 1)], dr[b * n_q:(b + 1) * n_q], par2[b],
                               1, n_q, temperature, ua2[b:b + 1], ub2[b:b + 1]) for b in range(B)]
        return tuple(np.concatenate([p[i] for p in parts]) for i in range(4))
    par = None if parent is None else _i32(parent)
    ua, ub = _f64(u_accept).reshape(B, max(n_q, 0)), _f64(u_bonus)
    alen = np.empty(B, dtype=np.int32)
    path = np.empty((B, n_q), dtype=np.int32)
    bonus = np.empty(B, dtype=np.int32)
    margin = np.empty(B, dtype=np.float64)
    rc = lib.oracle_accept_sample(_ptr(lg, _dp), _ptr(dr, _ip), _ptr(par, _ip), ctypes.c_int(B),
                                  ctypes.c_int(n_q), ctypes.c_int64(V), ctypes.c_double(temperature),
                                  _ptr(ua, _dp), _ptr(ub, _dp), _ptr(alen, _ip), _ptr(path, _ip),
                                  _ptr(bonus, _ip), _ptr(margin, _dp))
    if rc != 0:
        raise ValueError(f"oracle_accept_sample: bad arguments ({rc})")
    return alen, path, bonus, margin


def accept_sample_q(lg, draft_ids, parent, B: int, n_q: int, temperature: float, draft_q,
                    u_accept, u_bonus):
    """Stochastic acceptance against a sampled draft: draft_q [B*(n_q+1), V] holds, per logit row,
    the distribution its children's tokens were drawn from.  Returns (accept_len [B],
    accept_path [B, n_q], bonus_id [B], margin [B]).  parent [n_q], [B, n_q] or None."""
    lib = _load()
    lg, dq = _f64(lg), _f64(draft_q)
    V = lg.shape[1]
    assert lg.shape[0] == B * (n_q + 1) and dq.shape == lg.shape
    dr = _i32(draft_ids)
    if parent is not None and np.ndim(parent) == 2:      # one tree per sequence: per-sequence walks
        par2 = _i32(parent)
        assert par2.shape == (B, n_q)
        ua2, ub2 = np.asarray(u_accept).reshape(B, n_q), np.asarray(u_bonus).reshape(B)
        parts = [accept_sample_q(lg[b * (n_q + 1):(b + 1) * (n_q + 1)], dr[b * n_q:(b + 1) * n_q], par2[b],
                                 1, n_q, temperature, dq[b * (n_q + 1):(b + 1) * (n_q + 1)],
                                 ua2[b:b + 1], ub2[b:b + 1]) for b in range(B)]
        return tuple(np.concatenate([p[i] for p in parts]) for i in range(4))
    par = None if parent is None else _i32(parent)
    ua, ub = _f64(u_accept).reshape(B, max(n_q, 0)), _f64(u_bonus)
    alen = np.empty(B, dtype=np.int32)
    path = np.empty((B, n_q), dtype=np.int32)
    bonus = np.empty(B, dtype=np.int32)
    margin = np.empty(B, dtype=np.float64)
    rc = lib.oracle_accept_sample_q(_ptr(lg, _dp), _ptr(dr, _ip), _ptr(par, _ip), ctypes.c_int(B),
                                    ctypes.c_int(n_q), ctypes.c_int64(V), ctypes.c_double(temperature),
                                    _ptr(dq, _dp), _ptr(ua, _dp), _ptr(ub, _dp), _ptr(alen, _ip),
                                    _ptr(path, _ip), _ptr(bonus, _ip), _ptr(margin, _dp))
    if rc != 0:
        raise ValueError(f"oracle_accept_sample_q: bad arguments ({rc})")
    return alen, path, bonus, margin


def philox4x32_10(counter, key) -> np.ndarray:
    """One block of Philox4x32-10: counter 4 x uint32, key 2 x uint32 -> 4 x uint32."""
    c = np.ascontiguousarray(counter, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    assert c.shape == (4,) and k.shape == (2,)
    out = np.empty(4, dtype=np.uint32)
    up = ctypes.POINTER(ctypes.c_uint32)
    _load().oracle_philox4x32_10(c.ctypes.data_as(up), k.ctypes.data_as(up), out.ctypes.data_as(up))
    return out


def philox_uniforms(seed: int, offset: int, B: int, n_q: int):
    """The uniforms of a call that leaves their generation to the library: (u_accept [B, n_q],
    u_bonus [B]) float64, each a multiple of 2^-24 in [0, 1)."""
    ua = np.empty((B, max(n_q, 0)), dtype=np.float64)
    ub = np.empty(B, dtype=np.float64)
    _load().oracle_philox_uniforms(ctypes.c_uint64(seed), ctypes.c_uint64(offset), ctypes.c_int(B),
                                   ctypes.c_int(n_q), _ptr(ua, _dp), _ptr(ub, _dp))
    return ua, ub


def accept_sample_step(hidden, lm_head, draft_ids, parent, B: int, n_q: int, temperature: float,
                       u_accept, u_bonus):
    """lm_head GEMM + stochastic acceptance, as one step."""
    lg = logits(hidden, lm_head)
    alen, path, bonus, margin = accept_sample(lg, draft_ids, parent, B, n_q, temperature,
                                              u_accept, u_bonus)
    return {"accept_len": alen, "accept_path": path, "bonus_id": bonus, "margin": margin}


def topk_logprob(lg, k: int):
    """Per row: ids [M,k] of the k largest logits (decreasing, ties to the lower id), their
    log-softmax values [M,k], and the conditioning margin [M]."""
    lib = _load()
    lg = _f64(lg)
    M, V = lg.shape
    ids = np.empty((M, k), dtype=np.int32)
    logp = np.empty((M, k), dtype=np.float64)
    margin = np.empty(M, dtype=np.float64)
    lib.oracle_topk_logprob(_ptr(lg, _dp), ctypes.c_int(M), ctypes.c_int64(V), ctypes.c_int(k),
                            _ptr(ids, _ip), _ptr(logp, _dp), _ptr(margin, _dp))
    return ids, logp, margin


class TreePool:
    """Pool of draft-tree candidates grown level by level (see oracle_tree_expand)."""

    def __init__(self, width: int, depth: int):
        cap = width + max(depth - 1, 0) * width * width
        self.width, self.depth = width, depth
        self.tok = np.zeros(cap, dtype=np.int32)
        self.par = np.zeros(cap, dtype=np.int32)
        self.score = np.zeros(cap, dtype=np.float64)
        self.n = 0
        self.front = None            # pool indices of the current frontier (None = root)
        self.margin = np.inf

    def expand(self, cand_ids, cand_logp):
        lib = _load()
        ci, cl = _i32(cand_ids), _f64(cand_logp)
        n_front = 1 if self.front is None else len(self.front)
        assert ci.shape == (n_front, self.width) and cl.shape == ci.shape
        fin = None if self.front is None else _i32(self.front)
        fout = np.empty(self.width, dtype=np.int32)
        mg = ctypes.c_double(0.0)
        self.n = lib.oracle_tree_expand(ctypes.c_int(n_front), ctypes.c_int(self.width),
                                        _ptr(fin, _ip), _ptr(ci, _ip), _ptr(cl, _dp),
                                        _ptr(self.tok, _ip), _ptr(self.par, _ip),
                                        _ptr(self.score, _dp), ctypes.c_int(self.n),
                                        _ptr(fout, _ip), ctypes.byref(mg))
        self.front = fout
        self.margin = min(self.margin, mg.value)
        return fout

    def select(self, total: int):
        lib = _load()
        keep = min(total, self.n)
        parent = np.empty(keep, dtype=np.int32)
        ids = np.empty(keep, dtype=np.int32)
        pidx = np.empty(keep, dtype=np.int32)
        mg = ctypes.c_double(0.0)
        rc = lib.oracle_tree_select(_ptr(self.tok, _ip), _ptr(self.par, _ip), _ptr(self.score, _dp),
                                    ctypes.c_int(self.n), ctypes.c_int(total), _ptr(parent, _ip),
                                    _ptr(ids, _ip), _ptr(pidx, _ip), ctypes.byref(mg))
        if rc < 0:
            raise ValueError("kept set is not closed under ancestors")
        self.margin = min(self.margin, mg.value)
        return parent, ids, pidx
