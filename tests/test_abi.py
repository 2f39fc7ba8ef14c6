"""The C-ABI library: it loads, exports every symbol include/sparrow.h declares, and validates its
host-side arguments before touching the device (CPU only: no kernel is launched here)."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "sparrow.h")
LIB = os.path.join(ROOT, "paper_2602_15318_amd", "libsparrow.so")

OK, INVALID, UNSUPPORTED, WORKSPACE = 0, -1, -2, -3


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2602_15318_amd import build
        build.build()
    L = ctypes.CDLL(LIB)
    L.sparrow_last_error.restype = ctypes.c_char_p
    L.sparrow_version.restype = ctypes.c_char_p
    for f in ("sparrow_draft_window_attn_workspace", "sparrow_verify_attn_workspace",
              "sparrow_accept_workspace", "sparrow_accept_sample_workspace",
              "sparrow_draft_topk_workspace"):
        getattr(L, f).restype = ctypes.c_size_t
    return L


class Desc(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("scale", ctypes.c_float), ("kv_stride_token", ctypes.c_int64),
                ("kv_stride_head", ctypes.c_int64), ("parent_stride", ctypes.c_int32)]


def desc(dtype=1, hq=28, hkv=4, d=128, scale=0.0, st=None, sh=None):
    return Desc(dtype, hq, hkv, d, scale, hkv * d if st is None else st, d if sh is None else sh, 0)


def test_every_declared_symbol_is_exported(lib):
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)     # declarations only
    names = set(re.findall(r"\b(sparrow_[a-z_]+)\s*\(", text))
    assert {"sparrow_draft_window_attn", "sparrow_verify_attn", "sparrow_accept"} <= names
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} declared in sparrow.h but not exported"
    assert lib.sparrow_version().decode().count(".") == 1


P = ctypes.c_void_p(0x10000)        # fake, aligned, never dereferenced: validation fails first
i32 = ctypes.c_int32


def _cu(*v):
    a = np.array(v, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def test_verify_argument_validation(lib):
    cu, cup = _cu(0, 100)
    args = lambda d, B=1, n_q=4, ws=None, wsb=0: (ctypes.byref(d), P, P, P, cup, None, i32(B),
                                                   i32(n_q), P, None, ws, ctypes.c_size_t(wsb), None)
    assert lib.sparrow_verify_attn(None, P, P, P, cup, None, 1, 4, P, None, None, 0, None) == INVALID
    assert lib.sparrow_verify_attn(*args(desc(dtype=7))) == UNSUPPORTED
    assert lib.sparrow_verify_attn(*args(desc(d=96))) == UNSUPPORTED
    assert lib.sparrow_verify_attn(*args(desc(hq=28, hkv=5))) == INVALID
    assert lib.sparrow_verify_attn(*args(desc(st=100))) == INVALID          # stride < Hkv*d
    assert lib.sparrow_verify_attn(*args(desc(scale=-1.0))) == INVALID
    assert lib.sparrow_verify_attn(*args(desc(), n_q=65)) == UNSUPPORTED
    assert lib.sparrow_verify_attn(*args(desc(), B=65)) == UNSUPPORTED
    assert lib.sparrow_verify_attn(*args(desc(), n_q=101)) == UNSUPPORTED
    cu2, cup2 = _cu(0, 3)
    assert lib.sparrow_verify_attn(ctypes.byref(desc()), P, P, P, cup2, None, 1, 4, P, None, None, 0,
                                   None) == INVALID                          # fewer rows than n_q
    assert b"fewer" in lib.sparrow_last_error()
    assert lib.sparrow_verify_attn(*args(desc())) == WORKSPACE               # NULL workspace
    assert b"workspace" in lib.sparrow_last_error()
    assert lib.sparrow_verify_attn(*args(desc(), ws=P, wsb=16)) == WORKSPACE
    # misaligned q
    assert lib.sparrow_verify_attn(ctypes.byref(desc()), ctypes.c_void_p(0x10008), P, P, cup, None, 1,
                                   4, P, None, P, 1 << 30, None) == INVALID
    # degenerate sizes are no-ops, also without a device
    assert lib.sparrow_verify_attn(*args(desc(), B=0)) == OK
    assert lib.sparrow_verify_attn(*args(desc(), n_q=0)) == OK
    assert lib.sparrow_last_error() == b""
    assert lib.sparrow_verify_attn_passes(*args(desc()), i32(0)) == INVALID


def test_draft_argument_validation(lib):
    cu, cup = _cu(0, 100)
    ct, ctp = _cu(0, 10)
    call = lambda d, cu_text=ctp, window=8, B=1: lib.sparrow_draft_window_attn(
        ctypes.byref(d), P, P, P, cup, P, cu_text, i32(B), i32(window), P, None, None, 0, None)
    assert call(desc(), window=0) == INVALID
    assert call(desc(d=256)) == UNSUPPORTED
    e, ep = _cu(0, 0)
    assert call(desc(), cu_text=ep) == INVALID and b"text" in lib.sparrow_last_error()
    big, bp = _cu(0, 101)
    assert call(desc(), cu_text=bp) == INVALID         # more text positions than tokens
    assert call(desc(), B=0) == OK
    assert lib.sparrow_draft_window_attn_workspace(ctypes.byref(desc()), 1, 512) == 0


def test_accept_argument_validation(lib):
    call = lambda dtype=1, B=1, n_q=8, H=3584, V=152064, ws=None, wsb=0: lib.sparrow_accept(
        i32(dtype), P, P, P, None, i32(B), i32(n_q), i32(H), i32(V), P, P, P, P, ws,
        ctypes.c_size_t(wsb), None)
    assert call(dtype=3) == UNSUPPORTED
    assert call(B=8, n_q=64) == UNSUPPORTED           # 520 logit rows > 512
    assert call(B=8, n_q=8) == WORKSPACE              # 72 rows: valid since the limit is 512
    assert call(H=3580) == UNSUPPORTED                # rows not multiples of 16 bytes
    assert call(V=0) == INVALID
    assert call() == WORKSPACE
    assert call(B=0) == OK


def test_workspace_queries(lib):
    d = desc()
    v = lib.sparrow_verify_attn_workspace(ctypes.byref(d), 1, 8, ctypes.c_int64(26120))
    # about one split per compute unit: 64 splits x 4 KV heads x 16.5 KB (fp16 partials, fp32 m/l)
    assert 64 * 4 * 16.5 * 1024 <= v < 5 * 2 ** 20
    # a 30-node tree has 210 rows per KV head: two workgroups of 128 rows per (split, KV head),
    # planned in whole groups per XCD: 32 splits x 4 heads x 4 units of 64 rows
    t = lib.sparrow_verify_attn_workspace(ctypes.byref(d), 1, 30, ctypes.c_int64(26142))
    assert 32 * 4 * 4 * 16.5 * 1024 <= t < 12 * 2 ** 20
    # a 25-node tree (175 rows): one workgroup of 192 rows per (split, KV head), 64 splits
    t25 = lib.sparrow_verify_attn_workspace(ctypes.byref(d), 1, 25, ctypes.c_int64(26137))
    assert 64 * 4 * 3 * 16.5 * 1024 <= t25 < 14 * 2 ** 20
    # K/V beyond 2 GB per call: the plain-ALU path with its own layout (fp32 [split, n_q, Hq, d])
    big = lib.sparrow_verify_attn_workspace(ctypes.byref(d), 8, 8, ctypes.c_int64(3_000_000))
    assert big > 0 and big % 256 == 0
    assert lib.sparrow_verify_attn_workspace(ctypes.byref(d), 0, 8, ctypes.c_int64(26120)) == 0
    f32 = desc(dtype=0, hq=4, hkv=1, d=64)
    assert lib.sparrow_verify_attn_workspace(ctypes.byref(f32), 1, 4, ctypes.c_int64(516)) > 0
    a = lib.sparrow_accept_workspace(1, 1, 8, 3584, 152064)
    assert 0 < a < 2 ** 20
    assert lib.sparrow_accept_workspace(0, 1, 4, 256, 1024) > 0


def test_draft_input_argument_validation(lib):
    fc = lambda dtype=1, M=1, H=3584, V=1000, emb=P, tok=P: lib.sparrow_hsr_fc(
        i32(dtype), emb, tok, P, P, None, i32(M), i32(H), i32(V), P, None)
    assert fc(dtype=5) == UNSUPPORTED
    assert fc(M=65) == UNSUPPORTED and b"65" in lib.sparrow_last_error()
    assert fc(H=3580) == UNSUPPORTED
    assert fc(V=0) == INVALID
    assert fc(emb=None) == INVALID
    assert fc(emb=ctypes.c_void_p(0x10004)) == INVALID
    assert fc(M=0) == OK
    rows, rp = _cu(5, 9)
    qkv = lambda d, M=2, H=3584, eps=1e-6, kv=rp, cos=P: lib.sparrow_draft_qkv_append(
        ctypes.byref(d), P, P, ctypes.c_float(eps), P, None, cos, P, kv, i32(M), i32(H), P, P, P, None)
    assert qkv(desc(d=96)) == UNSUPPORTED
    assert qkv(desc(), M=65) == UNSUPPORTED
    assert qkv(desc(), eps=-1.0) == INVALID
    assert qkv(desc(), cos=None) == INVALID
    assert qkv(desc(), cos=ctypes.c_void_p(0x10004)) == INVALID
    dup, dp_ = _cu(7, 7)
    assert qkv(desc(), kv=dp_) == INVALID and b"same cache row" in lib.sparrow_last_error()
    neg, np_ = _cu(3, -2)
    assert qkv(desc(), kv=np_) == INVALID
    assert qkv(desc(), M=0) == OK


def test_commit_argument_validation(lib):
    cu, cup = _cu(0, 50)
    ptrs = (ctypes.c_void_p * 2)(0x10000, 0x20000)
    call = lambda d, nl=2, B=1, n_q=8, cu_=cup, hid=None, H=0, nxt=None, k=ptrs: lib.sparrow_kv_commit(
        ctypes.byref(d), k, ptrs, i32(nl), cu_, i32(B), i32(n_q), P, P, hid, i32(H), nxt, None)
    assert call(desc(), nl=65) == UNSUPPORTED
    assert call(desc(), B=65) == UNSUPPORTED
    assert call(desc(), n_q=65) == UNSUPPORTED
    short, sp_ = _cu(0, 5)
    assert call(desc(), cu_=sp_) == INVALID and b"fewer" in lib.sparrow_last_error()
    assert call(desc(), hid=P, H=3584) == INVALID          # next_hidden missing
    assert call(desc(), hid=P, H=3, nxt=P) == UNSUPPORTED  # rows not multiples of 16 bytes
    bad = (ctypes.c_void_p * 2)(0x10000, 0x20004)
    assert call(desc(), k=bad) == INVALID
    assert call(desc(), B=0) == OK
    assert call(desc(), nl=0) == OK


def test_accept_sample_and_tree_argument_validation(lib):
    samp = lambda T=1.0, V=152064, ws=None, wsb=0, ua=P: lib.sparrow_accept_sample(
        i32(1), P, P, P, None, i32(1), i32(8), i32(3584), i32(V), ctypes.c_float(T), ua, P, P, P, P,
        ws, ctypes.c_size_t(wsb), None)
    assert samp(T=0.0) == INVALID and b"temperature" in lib.sparrow_last_error()
    assert samp(T=float("inf")) == INVALID
    assert samp(V=(1 << 20) + 1) == UNSUPPORTED
    assert samp(ua=None) == INVALID
    assert samp() == WORKSPACE
    need = lib.sparrow_accept_sample_workspace(1, 1, 8, 3584, 152064)
    greedy = lib.sparrow_accept_workspace(1, 1, 8, 3584, 152064)
    assert need >= greedy + 9 * 152064 * 4                 # the stored logits
    topk = lambda M=8, k=8, V=152064, ws=None, wsb=0: lib.sparrow_draft_topk(
        i32(1), P, P, i32(M), i32(3584), i32(V), i32(k), P, P, ws, ctypes.c_size_t(wsb), None)
    assert topk(k=17) == UNSUPPORTED
    assert topk(k=0) == UNSUPPORTED
    assert topk(M=513) == UNSUPPORTED
    assert topk(V=300000) == UNSUPPORTED
    assert topk(V=4, k=8) == UNSUPPORTED                   # more tokens asked for than there are
    assert topk() == WORKSPACE
    assert topk(M=0) == OK
    assert lib.sparrow_draft_topk_workspace(1, 8, 3584, 152064, 8) > 8 * 152064 * 4
    exp = lambda nf=1, w=8, fin=None, npool=0: lib.sparrow_tree_expand(
        i32(nf), i32(w), fin, P, P, P, P, P, i32(npool), P, None)
    assert exp(w=17) == UNSUPPORTED
    assert exp(nf=17, fin=P) == UNSUPPORTED
    assert exp(nf=8, fin=P, npool=2040) == UNSUPPORTED     # pool capacity 2048
    assert exp(nf=2) == INVALID and b"level 0" in lib.sparrow_last_error()
    sel = lambda n=200, total=30: lib.sparrow_tree_select(P, P, P, i32(n), i32(total), P, P, P, None)
    assert sel(total=65) == UNSUPPORTED
    assert sel(n=2049) == UNSUPPORTED
    assert sel(n=0) == OK and sel(total=0) == OK


def test_stream_read_argument_validation(lib):
    lib.sparrow_stream_read.restype = ctypes.c_int
    call = lambda p, n, sink=P: lib.sparrow_stream_read(p, ctypes.c_size_t(n), sink, None)
    assert call(None, 0) == OK
    assert call(None, 64) == INVALID
    assert call(P, 40) == INVALID                          # not a multiple of 16
    assert call(ctypes.c_void_p(0x10004), 64) == INVALID   # misaligned
    assert call(P, 64, sink=None) == INVALID


def test_debug_validators_on_host_arrays(lib):
    """The synchronous precondition checks, given ordinary host memory (no device needed)."""
    ip = ctypes.POINTER(ctypes.c_int32)
    vp = lambda a: ctypes.c_void_p(a.ctypes.data)      # noqa: E731
    good = np.array([-1, 0, 0, 1, 3, -1], dtype=np.int32)
    assert lib.sparrow_debug_validate_parent(vp(good), 0, 1, 6, None) == OK
    assert lib.sparrow_debug_validate_parent(None, 0, 1, 6, None) == OK          # NULL = chain
    for bad_at, val in ((0, 0), (2, 2), (4, 7), (3, -2)):
        bad = good.copy()
        bad[bad_at] = val
        assert lib.sparrow_debug_validate_parent(vp(bad), 0, 1, 6, None) == INVALID
        assert f"parent[{bad_at}] = {val}".encode() in lib.sparrow_last_error()
    trees = np.full((3, 8), 99, dtype=np.int32)            # stride 8 > n_q = 6: padding is ignored
    trees[:, :6] = good
    assert lib.sparrow_debug_validate_parent(vp(trees), 8, 3, 6, None) == OK
    trees[2, 5] = 5
    assert lib.sparrow_debug_validate_parent(vp(trees), 8, 3, 6, None) == INVALID
    assert b"tree 2" in lib.sparrow_last_error()
    assert lib.sparrow_debug_validate_parent(vp(trees), 4, 3, 6, None) == INVALID    # stride < n_q
    cu = np.array([0, 10, 14], dtype=np.int32)
    ct = np.array([0, 3, 5], dtype=np.int32)
    tix = np.array([0, 4, 9, 1, 3], dtype=np.int32)
    call = lambda t, c=cu, x=ct: lib.sparrow_debug_validate_text_idx(                # noqa: E731
        vp(t), c.ctypes.data_as(ip), x.ctypes.data_as(ip), 2, None)
    assert call(tix) == OK
    for bad in ([0, 4, 10, 1, 3], [0, 4, 4, 1, 3], [4, 0, 9, 1, 3], [0, 4, 9, 1, 4], [-1, 4, 9, 1, 3]):
        assert call(np.array(bad, dtype=np.int32)) == INVALID, bad
    assert call(tix, x=np.array([0, 3, 3], dtype=np.int32)) == INVALID               # empty text domain
