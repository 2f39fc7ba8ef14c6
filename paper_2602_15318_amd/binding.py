"""ctypes binding of libsparrow.so: argument marshalling only.

Function names and argument order follow include/sparrow.h.  Tensors are torch tensors on the
GPU; the host arrays (cu_seqlens, cu_text) are numpy arrays / sequences of ints.  There is no
fallback: if the HIP library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsparrow.so")

SPARROW_F32 = 0
SPARROW_BF16 = 1


class SparrowError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"sparrow status {code}: {message}")
        self.code = code


class AttnDesc(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("scale", ctypes.c_float), ("kv_stride_token", ctypes.c_int64),
                ("kv_stride_head", ctypes.c_int64), ("parent_stride", ctypes.c_int32)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2602_15318_amd.build` "
            "(or __graft_entry__.build()); there is no fallback path")
    L = ctypes.CDLL(_LIB_PATH)
    vp, i32p, fp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32), ctypes.c_void_p
    dp = ctypes.POINTER(AttnDesc)
    L.sparrow_last_error.restype = ctypes.c_char_p
    L.sparrow_version.restype = ctypes.c_char_p
    L.sparrow_draft_window_attn_workspace.restype = ctypes.c_size_t
    L.sparrow_draft_window_attn_workspace.argtypes = [dp, ctypes.c_int32, ctypes.c_int32]
    L.sparrow_draft_window_attn.restype = ctypes.c_int
    L.sparrow_draft_window_attn.argtypes = [dp, vp, vp, vp, i32p, vp, i32p, ctypes.c_int32,
                                            ctypes.c_int32, vp, fp, vp, ctypes.c_size_t, vp]
    L.sparrow_verify_attn_workspace.restype = ctypes.c_size_t
    L.sparrow_verify_attn_workspace.argtypes = [dp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64]
    L.sparrow_verify_attn.restype = ctypes.c_int
    L.sparrow_verify_attn.argtypes = [dp, vp, vp, vp, i32p, vp, ctypes.c_int32, ctypes.c_int32,
                                      vp, fp, vp, ctypes.c_size_t, vp]
    L.sparrow_verify_attn_static.restype = ctypes.c_int
    L.sparrow_verify_attn_static.argtypes = [dp, vp, vp, vp, i32p, vp, ctypes.c_int32, ctypes.c_int32,
                                             vp, fp, vp]
    L.sparrow_verify_attn_passes.restype = ctypes.c_int
    L.sparrow_verify_attn_passes.argtypes = L.sparrow_verify_attn.argtypes + [ctypes.c_int32]
    L.sparrow_accept_workspace.restype = ctypes.c_size_t
    L.sparrow_accept_workspace.argtypes = [ctypes.c_int32] * 5
    L.sparrow_accept.restype = ctypes.c_int
    L.sparrow_accept.argtypes = [ctypes.c_int32, vp, vp, vp, vp, ctypes.c_int32, ctypes.c_int32,
                                 ctypes.c_int32, ctypes.c_int32, vp, vp, vp, vp, vp,
                                 ctypes.c_size_t, vp]
    L.sparrow_accept_trees.restype = ctypes.c_int
    L.sparrow_accept_trees.argtypes = [ctypes.c_int32, vp, vp, vp, vp, ctypes.c_int32, ctypes.c_int32,
                                       ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, vp,
                                       vp, ctypes.c_size_t, vp]
    L.sparrow_accept_sample_trees.restype = ctypes.c_int
    L.sparrow_accept_sample_trees.argtypes = [ctypes.c_int32, vp, vp, vp, vp, ctypes.c_int32,
                                              ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                              ctypes.c_int32, ctypes.c_float, vp, vp, vp, vp, vp, vp,
                                              ctypes.c_size_t, vp]
    L.sparrow_accept_sample_q.restype = ctypes.c_int
    L.sparrow_accept_sample_q.argtypes = [ctypes.c_int32, vp, vp, vp, vp, ctypes.c_int32,
                                          ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                          ctypes.c_int32, ctypes.c_float, vp, vp, vp,
                                          ctypes.c_uint64, ctypes.c_uint64, vp, vp, vp, vp,
                                          ctypes.c_size_t, vp]
    L.sparrow_hsr_fc.restype = ctypes.c_int
    L.sparrow_hsr_fc.argtypes = [ctypes.c_int32, vp, vp, vp, vp, vp, ctypes.c_int32, ctypes.c_int32,
                                 ctypes.c_int32, vp, vp]
    L.sparrow_draft_qkv_append.restype = ctypes.c_int
    L.sparrow_draft_qkv_append.argtypes = [dp, vp, vp, ctypes.c_float, vp, vp, vp, vp, i32p,
                                           ctypes.c_int32, ctypes.c_int32, vp, vp, vp, vp]
    L.sparrow_kv_commit.restype = ctypes.c_int
    L.sparrow_kv_commit.argtypes = [dp, ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_void_p),
                                    ctypes.c_int32, i32p, ctypes.c_int32, ctypes.c_int32, vp, vp,
                                    vp, ctypes.c_int32, vp, vp]
    L.sparrow_accept_sample_workspace.restype = ctypes.c_size_t
    L.sparrow_accept_sample_workspace.argtypes = [ctypes.c_int32] * 5
    L.sparrow_accept_sample.restype = ctypes.c_int
    L.sparrow_accept_sample.argtypes = [ctypes.c_int32, vp, vp, vp, vp, ctypes.c_int32, ctypes.c_int32,
                                        ctypes.c_int32, ctypes.c_int32, ctypes.c_float, vp, vp,
                                        vp, vp, vp, vp, ctypes.c_size_t, vp]
    L.sparrow_draft_topk_workspace.restype = ctypes.c_size_t
    L.sparrow_draft_topk_workspace.argtypes = [ctypes.c_int32] * 5
    L.sparrow_draft_topk.restype = ctypes.c_int
    L.sparrow_draft_topk.argtypes = [ctypes.c_int32, vp, vp, ctypes.c_int32, ctypes.c_int32,
                                     ctypes.c_int32, ctypes.c_int32, vp, vp, vp, ctypes.c_size_t, vp]
    L.sparrow_tree_expand.restype = ctypes.c_int
    L.sparrow_tree_expand.argtypes = [ctypes.c_int32, ctypes.c_int32, vp, vp, vp, vp, vp, vp,
                                      ctypes.c_int32, vp, vp]
    L.sparrow_tree_select.restype = ctypes.c_int
    L.sparrow_tree_select.argtypes = [vp, vp, vp, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, vp]
    L.sparrow_debug_validate_parent.restype = ctypes.c_int
    L.sparrow_debug_validate_parent.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp]
    L.sparrow_debug_validate_text_idx.restype = ctypes.c_int
    L.sparrow_debug_validate_text_idx.argtypes = [vp, i32p, i32p, ctypes.c_int32, vp]
    L.sparrow_stream_read.restype = ctypes.c_int
    L.sparrow_stream_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
    L.sparrow_stream_read_shape.restype = ctypes.c_int
    L.sparrow_stream_read_shape.argtypes = [vp, ctypes.c_size_t, vp, ctypes.c_int32, ctypes.c_int32,
                                            ctypes.c_int32, vp]
    return L


lib = _load()


def library_path() -> str:
    return _LIB_PATH


def version() -> str:
    return lib.sparrow_version().decode()


def last_error() -> str:
    return lib.sparrow_last_error().decode()


def _check(rc: int) -> None:
    if rc != 0:
        raise SparrowError(rc, last_error())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return SPARROW_F32
    if t.dtype == torch.bfloat16:
        return SPARROW_BF16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _host_i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.int32)


def _i32p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _parent_stride(parent: Optional[torch.Tensor], n_q: int, B: int) -> int:
    """0 for a tree [n_q] shared by all sequences, the row stride for per-sequence trees [B, n_q]."""
    if parent is None:
        return 0
    if parent.dtype != torch.int32:
        raise ValueError("parent must be an int32 tensor")
    if parent.dim() == 1 and parent.numel() == n_q and parent.is_contiguous():
        return 0
    if parent.dim() == 2 and tuple(parent.shape) == (B, n_q) and parent.stride(1) == 1 and n_q > 0:
        return int(parent.stride(0)) if B > 1 else n_q
    raise ValueError("parent must be int32 [n_q] (one tree for all sequences) or [B, n_q]")


def _desc(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, scale: float,
          parent_stride: int = 0) -> AttnDesc:
    if k.dim() != 3 or k.stride(2) != 1 or v.stride() != k.stride() or v.shape != k.shape:
        raise ValueError("k and v must be [T, Hkv, d] with identical strides and a contiguous d")
    if not q.is_contiguous():
        raise ValueError("q must be contiguous [rows, Hq, d]")
    return AttnDesc(_dtype_code(q), q.shape[1], k.shape[1], q.shape[2], float(scale),
                    k.stride(0), k.stride(1), int(parent_stride))


def _workspace(nbytes: int, device, workspace: Optional[torch.Tensor]) -> Optional[torch.Tensor]:
    if workspace is not None:
        return workspace
    if nbytes == 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def draft_window_attn(q, k, v, cu_seqlens, text_idx, cu_text, window: int, scale: float = 0.0,
                      out=None, lse=None, want_lse: bool = True, stream=None):
    """sparrow_draft_window_attn.  q [B,Hq,d]; k,v [T,Hkv,d]; text_idx int32 device tensor.
    Returns (out, lse)."""
    B = q.shape[0]
    d = _desc(q, k, v, scale)
    cu, ct = _host_i32(cu_seqlens), _host_i32(cu_text)
    if cu.shape != (B + 1,) or ct.shape != (B + 1,):
        raise ValueError("cu_seqlens and cu_text must have B+1 entries")
    if text_idx.dtype != torch.int32 or not text_idx.is_contiguous():
        raise ValueError("text_idx must be a contiguous int32 tensor")
    out = torch.empty_like(q) if out is None else out
    if lse is None and want_lse:
        lse = torch.empty(q.shape[:2], dtype=torch.float32, device=q.device)
    _check(lib.sparrow_draft_window_attn(ctypes.byref(d), _ptr(q), _ptr(k), _ptr(v), _i32p(cu),
                                         _ptr(text_idx), _i32p(ct), B, int(window), _ptr(out),
                                         _ptr(lse), None, 0, _stream_ptr(stream)))
    return out, lse


def verify_attn_workspace_bytes(q, k, v, B: int, n_q: int, total_tokens: int,
                                scale: float = 0.0) -> int:
    d = _desc(q, k, v, scale)
    return int(lib.sparrow_verify_attn_workspace(ctypes.byref(d), B, n_q, int(total_tokens)))


def verify_attn(q, k, v, cu_seqlens, parent, n_q: int, scale: float = 0.0, out=None, lse=None,
                want_lse: bool = True, workspace=None, stream=None, passes: int = 3):
    """sparrow_verify_attn (sparrow_verify_attn_passes when passes != 3).  q [B*n_q,Hq,d];
    k,v [sum(L_b+n_q),Hkv,d]; parent int32 device tensor [n_q] (one tree for all sequences),
    [B, n_q] (one tree per sequence) or None (chain).  Returns (out, lse)."""
    cu = _host_i32(cu_seqlens)
    B = cu.shape[0] - 1
    d = _desc(q, k, v, scale, _parent_stride(parent, n_q, B))
    out = torch.empty_like(q) if out is None else out
    if lse is None and want_lse:
        lse = torch.empty(q.shape[:2], dtype=torch.float32, device=q.device)
    need = int(lib.sparrow_verify_attn_workspace(ctypes.byref(d), B, n_q, int(cu[-1]) - int(cu[0]))) if B > 0 else 0
    ws = _workspace(need, q.device, workspace)
    args = (ctypes.byref(d), _ptr(q), _ptr(k), _ptr(v), _i32p(cu), _ptr(parent), B, int(n_q),
            _ptr(out), _ptr(lse), _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(),
            _stream_ptr(stream))
    if passes == 3:
        _check(lib.sparrow_verify_attn(*args))
    else:
        _check(lib.sparrow_verify_attn_passes(*args, int(passes)))
    return out, lse


STATIC_WS_BYTES = 16 * 1024 * 1024      # SPARROW_STATIC_WS_BYTES


def verify_attn_static(q, k, v, cu_seqlens, parent, n_q: int, out, lse=None, scale: float = 0.0,
                       stream=None):
    """sparrow_verify_attn_static: the verification attention on the library's own scratch.  The
    caller passes every output; nothing is allocated here or in the library."""
    cu = _host_i32(cu_seqlens)
    B = cu.shape[0] - 1
    d = _desc(q, k, v, scale, _parent_stride(parent, n_q, B))
    _check(lib.sparrow_verify_attn_static(ctypes.byref(d), _ptr(q), _ptr(k), _ptr(v), _i32p(cu),
                                          _ptr(parent), B, int(n_q), _ptr(out), _ptr(lse),
                                          _stream_ptr(stream)))
    return out, lse


def accept_workspace_bytes(dtype_code: int, B: int, n_q: int, hidden: int, vocab: int) -> int:
    return int(lib.sparrow_accept_workspace(dtype_code, B, n_q, hidden, vocab))


def accept(hidden_rows, lm_head, draft_ids, parent, B: int, n_q: int, workspace=None,
           outputs=None, stream=None):
    """sparrow_accept.  hidden_rows [B*(n_q+1), H]; lm_head [V, H]; draft_ids int32 [B*n_q].
    Returns a dict of int32 device tensors: target_ids, accept_len, accept_path, bonus_id."""
    if not hidden_rows.is_contiguous() or not lm_head.is_contiguous():
        raise ValueError("hidden_rows and lm_head must be contiguous")
    if hidden_rows.dtype != lm_head.dtype:
        raise ValueError("hidden_rows and lm_head must share a dtype")
    H, V = hidden_rows.shape[1], lm_head.shape[0]
    if hidden_rows.shape[0] != B * (n_q + 1) or lm_head.shape[1] != H:
        raise ValueError("shape mismatch between hidden_rows, lm_head, B and n_q")
    dev = hidden_rows.device
    code = _dtype_code(hidden_rows)
    if outputs is None:
        outputs = {"target_ids": torch.empty(B * (n_q + 1), dtype=torch.int32, device=dev),
                   "accept_len": torch.empty(B, dtype=torch.int32, device=dev),
                   "accept_path": torch.empty(B, max(n_q, 1), dtype=torch.int32, device=dev)[:, :n_q],
                   "bonus_id": torch.empty(B, dtype=torch.int32, device=dev)}
    ws = _workspace(accept_workspace_bytes(code, B, n_q, H, V), dev, workspace)
    path = outputs["accept_path"]
    if n_q > 0 and not path.is_contiguous():
        raise ValueError("accept_path must be contiguous")
    _check(lib.sparrow_accept_trees(code, _ptr(hidden_rows), _ptr(lm_head), _ptr(draft_ids),
                              _ptr(parent), _parent_stride(parent, n_q, B), B, n_q, H, V,
                              _ptr(outputs["target_ids"]),
                              _ptr(outputs["accept_len"]), _ptr(path) if n_q > 0 else None,
                              _ptr(outputs["bonus_id"]), _ptr(ws),
                              0 if ws is None else ws.numel() * ws.element_size(),
                              _stream_ptr(stream)))
    return outputs


def hsr_fc(embed, token_ids, h_prev, w_fc, b_fc=None, out=None, stream=None):
    """sparrow_hsr_fc: z = FC(embed[token_ids] (+) h_prev).  embed [V,H]; token_ids int32 [M];
    h_prev [M,H]; w_fc [H,2H]; b_fc [H] or None.  Returns z [M,H]."""
    M, H = h_prev.shape
    for t in (embed, h_prev, w_fc) + (() if b_fc is None else (b_fc,)):
        if not t.is_contiguous() or t.dtype != h_prev.dtype:
            raise ValueError("embed, h_prev, w_fc and b_fc must be contiguous and of one dtype")
    if embed.shape[1] != H or tuple(w_fc.shape) != (H, 2 * H):
        raise ValueError("embed must be [V, H] and w_fc [H, 2H]")
    if token_ids.dtype != torch.int32 or token_ids.shape != (M,) or not token_ids.is_contiguous():
        raise ValueError("token_ids must be a contiguous int32 tensor of M entries")
    out = torch.empty_like(h_prev) if out is None else out
    _check(lib.sparrow_hsr_fc(_dtype_code(h_prev), _ptr(embed), _ptr(token_ids), _ptr(h_prev),
                              _ptr(w_fc), _ptr(b_fc), M, H, embed.shape[0], _ptr(out),
                              _stream_ptr(stream)))
    return out


def draft_qkv_append(z, norm_weight, eps: float, w_qkv, b_qkv, rope_cos, rope_sin, kv_rows,
                     n_q_heads: int, k_cache, v_cache, q_out=None, stream=None):
    """sparrow_draft_qkv_append.  z [M,H]; w_qkv [(Hq+2Hkv)d, H]; rope_cos/sin float32 [M,d/2];
    kv_rows host int32 [M]; k_cache, v_cache [T,Hkv,d] (written in place).  Returns q [M,Hq,d]."""
    M, H = z.shape
    Hkv, d = k_cache.shape[1], k_cache.shape[2]
    if k_cache.stride(2) != 1 or v_cache.stride() != k_cache.stride() or v_cache.shape != k_cache.shape:
        raise ValueError("k_cache and v_cache must be [T, Hkv, d] with identical strides and a contiguous d")
    for t in (z, norm_weight, w_qkv) + (() if b_qkv is None else (b_qkv,)):
        if not t.is_contiguous() or t.dtype != z.dtype:
            raise ValueError("z, norm_weight, w_qkv and b_qkv must be contiguous and of one dtype")
    if tuple(w_qkv.shape) != ((n_q_heads + 2 * Hkv) * d, H):
        raise ValueError("w_qkv must be [(Hq + 2 Hkv) d, H]")
    for t in (rope_cos, rope_sin):
        if t.dtype != torch.float32 or tuple(t.shape) != (M, d // 2) or not t.is_contiguous():
            raise ValueError("rope_cos and rope_sin must be contiguous float32 [M, d/2]")
    rows = _host_i32(kv_rows)
    if rows.shape != (M,):
        raise ValueError("kv_rows must have M entries")
    q_out = torch.empty((M, n_q_heads, d), dtype=z.dtype, device=z.device) if q_out is None else q_out
    desc = AttnDesc(_dtype_code(z), n_q_heads, Hkv, d, 0.0, k_cache.stride(0), k_cache.stride(1))
    _check(lib.sparrow_draft_qkv_append(ctypes.byref(desc), _ptr(z), _ptr(norm_weight), float(eps),
                                        _ptr(w_qkv), _ptr(b_qkv), _ptr(rope_cos), _ptr(rope_sin),
                                        _i32p(rows), M, H, _ptr(q_out), _ptr(k_cache),
                                        _ptr(v_cache), _stream_ptr(stream)))
    return q_out


def kv_commit(k_layers, v_layers, cu_seqlens, n_q: int, accept_path, accept_len, hidden_rows=None,
              next_hidden=None, stream=None):
    """sparrow_kv_commit.  k_layers, v_layers: lists of [T,Hkv,d] tensors (moved in place);
    accept_path int32 [B,n_q] and accept_len int32 [B] device tensors.  Returns next_hidden
    ([B,H], or None without hidden_rows)."""
    cu = _host_i32(cu_seqlens)
    B = cu.shape[0] - 1
    nl = len(k_layers)
    if len(v_layers) != nl:
        raise ValueError("k_layers and v_layers must have the same length")
    for t in (accept_path, accept_len):
        if t.dtype != torch.int32 or not t.is_contiguous():
            raise ValueError("accept_path and accept_len must be contiguous int32 tensors")
    ref = k_layers[0] if nl else None
    for t in list(k_layers) + list(v_layers):
        if t.dim() != 3 or t.stride(2) != 1 or t.stride() != ref.stride() or t.dtype != ref.dtype:
            raise ValueError("every layer's K and V must be [T, Hkv, d] with the same strides and dtype")
    if ref is not None:
        desc = AttnDesc(_dtype_code(ref), ref.shape[1], ref.shape[1], ref.shape[2], 0.0,
                        ref.stride(0), ref.stride(1))
    else:
        d0 = hidden_rows
        desc = AttnDesc(_dtype_code(d0), 1, 1, 64, 0.0, 64, 64)
    kp = (ctypes.c_void_p * max(nl, 1))(*[t.data_ptr() for t in k_layers])
    vp_ = (ctypes.c_void_p * max(nl, 1))(*[t.data_ptr() for t in v_layers])
    H = 0
    if hidden_rows is not None:
        if not hidden_rows.is_contiguous():
            raise ValueError("hidden_rows must be contiguous")
        H = hidden_rows.shape[1]
        if next_hidden is None:
            next_hidden = torch.empty((B, H), dtype=hidden_rows.dtype, device=hidden_rows.device)
    _check(lib.sparrow_kv_commit(ctypes.byref(desc), kp, vp_, nl, _i32p(cu), B, n_q,
                                 _ptr(accept_path), _ptr(accept_len), _ptr(hidden_rows), H,
                                 _ptr(next_hidden), _stream_ptr(stream)))
    return next_hidden


def accept_sample_workspace_bytes(dtype_code: int, B: int, n_q: int, hidden: int, vocab: int) -> int:
    return int(lib.sparrow_accept_sample_workspace(dtype_code, B, n_q, hidden, vocab))


def accept_sample(hidden_rows, lm_head, draft_ids, parent, B: int, n_q: int, temperature: float,
                  u_accept, u_bonus, workspace=None, outputs=None, stream=None):
    """sparrow_accept_sample.  u_accept float32 [B,n_q], u_bonus float32 [B] device tensors.
    Returns {"accept_len", "accept_path", "bonus_id"} (int32 device tensors)."""
    M, H = hidden_rows.shape
    V = lm_head.shape[0]
    if M != B * (n_q + 1) or lm_head.shape[1] != H:
        raise ValueError("hidden_rows must be [B*(n_q+1), H] and lm_head [V, H]")
    if not hidden_rows.is_contiguous() or not lm_head.is_contiguous() or lm_head.dtype != hidden_rows.dtype:
        raise ValueError("hidden_rows and lm_head must be contiguous and of one dtype")
    for t in (u_accept, u_bonus):
        if t.dtype != torch.float32 or not t.is_contiguous():
            raise ValueError("u_accept and u_bonus must be contiguous float32 tensors")
    dev = hidden_rows.device
    code = _dtype_code(hidden_rows)
    ws = _workspace(accept_sample_workspace_bytes(code, B, n_q, H, V), dev, workspace)
    if outputs is None:
        outputs = {"accept_len": torch.empty(B, dtype=torch.int32, device=dev),
                   "accept_path": torch.empty((B, n_q), dtype=torch.int32, device=dev),
                   "bonus_id": torch.empty(B, dtype=torch.int32, device=dev)}
    _check(lib.sparrow_accept_sample_trees(code, _ptr(hidden_rows), _ptr(lm_head), _ptr(draft_ids),
                                     _ptr(parent), _parent_stride(parent, n_q, B), B, n_q, H, V,
                                     float(temperature),
                                     _ptr(u_accept), _ptr(u_bonus), _ptr(outputs["accept_len"]),
                                     _ptr(outputs["accept_path"]) if n_q > 0 else None,
                                     _ptr(outputs["bonus_id"]), _ptr(ws),
                                     0 if ws is None else ws.numel(), _stream_ptr(stream)))
    return outputs


def accept_sample_q(hidden_rows, lm_head, draft_ids, parent, B: int, n_q: int, temperature: float,
                    draft_probs=None, u_accept=None, u_bonus=None, seed: int = 0, offset: int = 0,
                    workspace=None, outputs=None, stream=None):
    """sparrow_accept_sample_q: stochastic acceptance against a sampled draft (draft_probs float32
    [B*(n_q+1), V], or None for the deterministic-children rule), with the caller's uniforms or,
    if both are None, uniforms generated by the library from (seed, offset)."""
    M, H = hidden_rows.shape
    V = lm_head.shape[0]
    if M != B * (n_q + 1) or lm_head.shape[1] != H:
        raise ValueError("hidden_rows must be [B*(n_q+1), H] and lm_head [V, H]")
    if not hidden_rows.is_contiguous() or not lm_head.is_contiguous() or lm_head.dtype != hidden_rows.dtype:
        raise ValueError("hidden_rows and lm_head must be contiguous and of one dtype")
    for t in (u_accept, u_bonus, draft_probs):
        if t is not None and (t.dtype != torch.float32 or not t.is_contiguous()):
            raise ValueError("u_accept, u_bonus and draft_probs must be contiguous float32 tensors")
    if draft_probs is not None and tuple(draft_probs.shape) != (M, V):
        raise ValueError("draft_probs must be [B*(n_q+1), V]")
    dev = hidden_rows.device
    code = _dtype_code(hidden_rows)
    ws = _workspace(accept_sample_workspace_bytes(code, B, n_q, H, V), dev, workspace)
    if outputs is None:
        outputs = {"accept_len": torch.empty(B, dtype=torch.int32, device=dev),
                   "accept_path": torch.empty((B, n_q), dtype=torch.int32, device=dev),
                   "bonus_id": torch.empty(B, dtype=torch.int32, device=dev)}
    _check(lib.sparrow_accept_sample_q(code, _ptr(hidden_rows), _ptr(lm_head), _ptr(draft_ids),
                                       _ptr(parent), _parent_stride(parent, n_q, B), B, n_q, H, V,
                                       float(temperature), _ptr(draft_probs), _ptr(u_accept),
                                       _ptr(u_bonus), int(seed), int(offset),
                                       _ptr(outputs["accept_len"]),
                                       _ptr(outputs["accept_path"]) if n_q > 0 else None,
                                       _ptr(outputs["bonus_id"]), _ptr(ws),
                                       0 if ws is None else ws.numel(), _stream_ptr(stream)))
    return outputs


def draft_topk(hidden_rows, lm_head, k: int, workspace=None, stream=None):
    """sparrow_draft_topk: per row the k most likely tokens (int32 [M,k], decreasing) and their
    natural-log softmax values (float32 [M,k])."""
    M, H = hidden_rows.shape
    V = lm_head.shape[0]
    if lm_head.shape[1] != H or not hidden_rows.is_contiguous() or not lm_head.is_contiguous() \
            or lm_head.dtype != hidden_rows.dtype:
        raise ValueError("hidden_rows [M,H] and lm_head [V,H] must be contiguous and of one dtype")
    dev = hidden_rows.device
    code = _dtype_code(hidden_rows)
    ws = _workspace(int(lib.sparrow_draft_topk_workspace(code, M, H, V, k)), dev, workspace)
    ids = torch.empty((M, k), dtype=torch.int32, device=dev)
    logp = torch.empty((M, k), dtype=torch.float32, device=dev)
    _check(lib.sparrow_draft_topk(code, _ptr(hidden_rows), _ptr(lm_head), M, H, V, k, _ptr(ids),
                                  _ptr(logp), _ptr(ws), 0 if ws is None else ws.numel(),
                                  _stream_ptr(stream)))
    return ids, logp


class TreePool:
    """Device-side candidate pool of the dynamic draft tree (sparrow_tree_expand / _select)."""

    def __init__(self, width: int, depth: int, device="cuda"):
        cap = width + max(depth - 1, 0) * width * width
        self.width = width
        self.tok = torch.zeros(cap, dtype=torch.int32, device=device)
        self.par = torch.zeros(cap, dtype=torch.int32, device=device)
        self.score = torch.zeros(cap, dtype=torch.float32, device=device)
        self.n = 0
        self.front = None

    def expand(self, cand_ids, cand_logp, stream=None):
        n_front = 1 if self.front is None else self.front.shape[0]
        if tuple(cand_ids.shape) != (n_front, self.width) or cand_ids.dtype != torch.int32 \
                or cand_logp.dtype != torch.float32 or cand_logp.shape != cand_ids.shape \
                or not cand_ids.is_contiguous() or not cand_logp.is_contiguous():
            raise ValueError("cand_ids int32 / cand_logp float32 must be contiguous [n_front, width]")
        if self.n + n_front * self.width > self.tok.shape[0]:
            raise ValueError("pool is full: more levels than the depth it was sized for")
        out = torch.empty(self.width, dtype=torch.int32, device=self.tok.device)
        _check(lib.sparrow_tree_expand(n_front, self.width, _ptr(self.front), _ptr(cand_ids),
                                       _ptr(cand_logp), _ptr(self.tok), _ptr(self.par),
                                       _ptr(self.score), self.n, _ptr(out), _stream_ptr(stream)))
        self.n += n_front * self.width
        self.front = out
        return out

    def select(self, total: int, stream=None):
        keep = min(total, self.n)
        dev = self.tok.device
        parent = torch.empty(keep, dtype=torch.int32, device=dev)
        ids = torch.empty(keep, dtype=torch.int32, device=dev)
        pidx = torch.empty(keep, dtype=torch.int32, device=dev)
        _check(lib.sparrow_tree_select(_ptr(self.tok), _ptr(self.par), _ptr(self.score), self.n,
                                       total, _ptr(parent), _ptr(ids), _ptr(pidx),
                                       _stream_ptr(stream)))
        return parent, ids, pidx


def debug_validate_parent(parent: torch.Tensor, n_q: int, B: int = 1, stream=None) -> None:
    """sparrow_debug_validate_parent on a device tensor [n_q] or [B, n_q]: raises SparrowError
    naming the first entry outside [-1, i).  Synchronises the stream."""
    _check(lib.sparrow_debug_validate_parent(_ptr(parent), _parent_stride(parent, n_q, B), B, int(n_q),
                                             _stream_ptr(stream)))


def debug_validate_text_idx(text_idx: torch.Tensor, cu_seqlens, cu_text, stream=None) -> None:
    """sparrow_debug_validate_text_idx on a device tensor: per sequence strictly ascending,
    in range, not empty.  Synchronises the stream."""
    cu, ct = _host_i32(cu_seqlens), _host_i32(cu_text)
    if text_idx.dtype != torch.int32 or not text_idx.is_contiguous():
        raise ValueError("text_idx must be a contiguous int32 tensor")
    _check(lib.sparrow_debug_validate_text_idx(_ptr(text_idx), _i32p(cu), _i32p(ct), cu.shape[0] - 1,
                                               _stream_ptr(stream)))


def stream_read(t: torch.Tensor, sink: torch.Tensor, stream=None, shape=None) -> None:
    """sparrow_stream_read over the storage of a contiguous tensor (measurement aid); `shape` =
    (workgroups, loads_in_flight, regions) selects sparrow_stream_read_shape."""
    if not t.is_contiguous():
        raise ValueError("stream_read needs a contiguous tensor")
    nbytes = t.numel() * t.element_size()
    if shape is None:
        _check(lib.sparrow_stream_read(_ptr(t), nbytes, _ptr(sink), _stream_ptr(stream)))
    else:
        wgs, in_flight, regions = shape
        _check(lib.sparrow_stream_read_shape(_ptr(t), nbytes, _ptr(sink), int(wgs), int(in_flight),
                                             int(regions), _stream_ptr(stream)))
