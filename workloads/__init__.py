"""Seeded synthetic inputs for the Sparrow speculative-decoding hot path.

This module only *draws inputs*: Gaussian tensors, position-type layouts
(which context positions are text and which are visual), draft trees and
token ids.  It contains none of the method's arithmetic (no attention, no
softmax, no GEMM, no argmax, no acceptance) and is imported by the tests and
the benchmark to feed the very same bits to the CPU oracle and to the HIP
library (the rotary cos/sin rows of the draft's input side are drawn here too:
both sides receive them as inputs).  Neither of those two imports the other.

Shapes follow the five workload configurations C1..C5 (a tiny fp32 case, a
Qwen2.5-VL-7B-shaped single layer at 8k context, a 26k-context long-video
layer verified with a 60-node draft tree, a ragged batch of 8, and the full
28-layer verify step at 26k context).  The paper's evaluation videos and model
weights are not available; these inputs stand in for them and take only their
shapes: visual tokens dominate the context (Insight section: up to 25k visual
tokens, more than 99 % of the sequence) and text sits in a few short runs.

Every floating-point tensor is returned as a float32 numpy array whose values
are exactly representable in the case's storage type ("f32" or "bf16"), so
casting to that type on the device and widening to float64 for the oracle are
both lossless.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

TEXT = 0
VISUAL = 1


# --------------------------------------------------------------------------
# storage-type helpers (input preparation only)
# --------------------------------------------------------------------------
def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even) and return
    them as float32.  Finite inputs only."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return round_to_bf16(x)
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    raise ValueError(f"unknown storage type {dtype!r}")


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bf16-exact."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def _rng(seed: int, *stream: int) -> np.random.Generator:
    """Independent PCG64 stream per (seed, stream...) key."""
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, *stream])))


def _normal(rng: np.random.Generator, shape, dtype: str, std: float = 1.0) -> np.ndarray:
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return to_storage(x, dtype)


# --------------------------------------------------------------------------
# configurations
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Config:
    name: str
    dtype: str                      # storage type of q/k/v/hidden/lm_head
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    batch: int
    # one list of (type, run_length) per sequence; None = drawn at random (ragged)
    layout: Optional[Tuple[Tuple[Tuple[int, int], ...], ...]]
    window: int
    n_q: int                        # draft rows verified per sequence
    tree: bool                      # True: 60-node pruned tree, False: chain
    hidden: int
    vocab: int
    n_layers: int = 1

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


C1 = Config("C1", "f32", 4, 1, 64, 1,
            (((TEXT, 16), (VISUAL, 448), (TEXT, 48)),), 32, 4, False, 256, 1024)
C2 = Config("C2", "bf16", 28, 4, 128, 1,
            (((TEXT, 256), (VISUAL, 7680), (TEXT, 256)),), 256, 5, False, 3584, 152064)
C3 = Config("C3", "bf16", 28, 4, 128, 1,
            (((TEXT, 512), (VISUAL, 25088), (TEXT, 512)),), 512, 60, True, 3584, 152064)
C4 = Config("C4", "bf16", 28, 4, 128, 8, None, 256, 6, False, 3584, 152064)
C5 = Config("C5", "bf16", 28, 4, 128, 1,
            (((TEXT, 512), (VISUAL, 25088), (TEXT, 512)),), 512, 8, False, 3584, 152064,
            n_layers=28)
CONFIGS = {c.name: c for c in (C1, C2, C3, C4, C5)}


# --------------------------------------------------------------------------
# position-type layouts
# --------------------------------------------------------------------------
def _composition(rng: np.random.Generator, total: int, parts: int) -> List[int]:
    """Random composition of `total` into `parts` positive integers."""
    if parts == 1:
        return [total]
    cuts = np.sort(rng.choice(np.arange(1, total), size=parts - 1, replace=False))
    edges = np.concatenate(([0], cuts, [total]))
    return [int(b - a) for a, b in zip(edges[:-1], edges[1:])]


def ragged_layouts(seed: int, batch: int = 8, lo: int = 4096, hi: int = 16384
                   ) -> Tuple[Tuple[Tuple[int, int], ...], ...]:
    """C4 layouts: context length uniform in [lo, hi], visual fraction uniform
    in [0.85, 0.97], text in 1-4 contiguous runs, the last run ending at the
    final position (the position the draft query sits at)."""
    rng = _rng(seed, 401)
    layouts = []
    for _ in range(batch):
        L = int(rng.integers(lo, hi + 1))
        vf = float(rng.uniform(0.85, 0.97))
        n_seg = int(rng.integers(1, 5))
        n_vis = min(L - n_seg, max(n_seg, int(round(L * vf))))
        n_text = L - n_vis
        text_runs = _composition(rng, n_text, n_seg)
        # n_seg == 1: [visual][text]; otherwise text and visual alternate,
        # starting and ending with text.
        n_gaps = 1 if n_seg == 1 else n_seg - 1
        vis_runs = _composition(rng, n_vis, n_gaps)
        runs: List[Tuple[int, int]] = []
        if n_seg == 1:
            runs = [(VISUAL, vis_runs[0]), (TEXT, text_runs[0])]
        else:
            for i in range(n_seg):
                runs.append((TEXT, text_runs[i]))
                if i < n_gaps:
                    runs.append((VISUAL, vis_runs[i]))
        layouts.append(tuple(runs))
    return tuple(layouts)


def layouts_of(cfg: Config, seed: int):
    return cfg.layout if cfg.layout is not None else ragged_layouts(seed, cfg.batch)


def layout_length(layout) -> int:
    return int(sum(n for _, n in layout))


def position_types(layout) -> np.ndarray:
    """int8 [L]: TEXT or VISUAL for every context position."""
    return np.concatenate([np.full(n, t, dtype=np.int8) for t, n in layout])


def text_index(layout) -> np.ndarray:
    """Ascending int32 positions of the text tokens (the text domain)."""
    return np.flatnonzero(position_types(layout) == TEXT).astype(np.int32)


# --------------------------------------------------------------------------
# draft trees
# --------------------------------------------------------------------------
def chain_parent(n_q: int) -> np.ndarray:
    return np.arange(-1, n_q - 1, dtype=np.int32)


def pruned_tree(seed: int, n_nodes: int = 60,
                branching: Sequence[int] = (4, 3, 2, 2, 1, 1)) -> np.ndarray:
    """Parent array of a draft tree kept to a node budget, the way a
    dynamic-tree drafter reranks to "total tokens" (Experiment section, tree
    configurations total-depth-width): build the full tree with the given
    per-level branching, score every node by the product of uniform draws along
    its path, keep the `n_nodes` best (ancestor-closed, because a child never
    outscores its parent), make sure one path reaches full depth, and renumber
    so that parent[i] < i (level by level).  parent = -1 marks children of the
    last accepted token (the root, which is not a node)."""
    rng = _rng(seed, 301)
    par: List[int] = []
    score: List[float] = []
    depth: List[int] = []
    frontier = [-1]
    for lvl, br in enumerate(branching):
        nxt = []
        for p in frontier:
            for _ in range(br):
                s = float(rng.uniform(0.0, 1.0)) * (score[p] if p >= 0 else 1.0)
                par.append(p)
                score.append(s)
                depth.append(lvl + 1)
                nxt.append(len(par) - 1)
        frontier = nxt
    total = len(par)
    n_nodes = min(n_nodes, total)
    # forced full-depth path: from the best leaf of the deepest level upwards
    deepest = [i for i in range(total) if depth[i] == len(branching)]
    leaf = max(deepest, key=lambda i: score[i])
    forced = set()
    x = leaf
    while x >= 0:
        forced.add(x)
        x = par[x]
    order = sorted((i for i in range(total) if i not in forced), key=lambda i: -score[i])
    keep = set(forced)
    for i in order:
        if len(keep) >= n_nodes:
            break
        keep.add(i)  # ancestor-closed: ancestors have strictly larger score, hence earlier
    # ancestors of kept nodes are kept (scores are monotone), assert it anyway
    for i in keep:
        assert par[i] < 0 or par[i] in keep
    kept = sorted(keep, key=lambda i: (depth[i], i))
    new_id = {old: new for new, old in enumerate(kept)}
    parent = np.array([new_id[par[i]] if par[i] >= 0 else -1 for i in kept], dtype=np.int32)
    assert all(parent[i] < i for i in range(len(parent)))
    return parent


def parent_of(cfg: Config, seed: int) -> Optional[np.ndarray]:
    return pruned_tree(seed, cfg.n_q) if cfg.tree else None


# --------------------------------------------------------------------------
# cases
# --------------------------------------------------------------------------
@dataclass
class DraftCase:
    """Inputs of the draft model's text-anchored window attention: one query
    per sequence, the draft layer's K/V indexed by absolute position, and the
    ascending text-position index of every sequence (packed)."""
    cfg: Config
    q: np.ndarray            # [B, Hq, d]
    k: np.ndarray            # [T, Hkv, d], T = sum L_b
    v: np.ndarray
    cu_seqlens: np.ndarray   # int32 [B+1]
    text_idx: np.ndarray     # int32, sequence-local positions, packed
    cu_text: np.ndarray      # int32 [B+1]
    window: int
    types: List[np.ndarray] = field(default_factory=list)


@dataclass
class VerifyCase:
    """Inputs of the target's verification attention for one layer: n_q draft
    rows per sequence against that sequence's L_b context rows followed by the
    n_q draft rows themselves."""
    cfg: Config
    q: np.ndarray            # [B*n_q, Hq, d]
    k: np.ndarray            # [sum (L_b + n_q), Hkv, d]
    v: np.ndarray
    cu_seqlens: np.ndarray   # int32 [B+1], sequence b owns L_b + n_q rows
    parent: Optional[np.ndarray]
    n_q: int


@dataclass
class AcceptCase:
    cfg: Config
    hidden: np.ndarray       # [B*(n_q+1), H]
    lm_head: np.ndarray      # [V, H]
    draft_ids: np.ndarray    # int32 [B*n_q]
    parent: Optional[np.ndarray]
    n_q: int
    planted_ids: Optional[np.ndarray] = None   # int32 [B*(n_q+1)] when planted


def draft_case(cfg: Config, seed: int = 0, peaked: bool = False,
               layouts=None, window: Optional[int] = None) -> DraftCase:
    layouts = layouts if layouts is not None else layouts_of(cfg, seed)
    B = len(layouts)
    lens = [layout_length(l) for l in layouts]
    cu = np.concatenate(([0], np.cumsum(lens))).astype(np.int32)
    tidx = [text_index(l) for l in layouts]
    cu_text = np.concatenate(([0], np.cumsum([len(t) for t in tidx]))).astype(np.int32)
    rng = _rng(seed, 101)
    T = int(cu[-1])
    q = _normal(rng, (B, cfg.n_q_heads, cfg.head_dim), cfg.dtype, 4.0 if peaked else 1.0)
    k = _normal(rng, (T, cfg.n_kv_heads, cfg.head_dim), cfg.dtype)
    v = _normal(rng, (T, cfg.n_kv_heads, cfg.head_dim), cfg.dtype)
    return DraftCase(cfg, q, k, v, cu, np.concatenate(tidx).astype(np.int32), cu_text,
                     cfg.window if window is None else window,
                     [position_types(l) for l in layouts])


def verify_case(cfg: Config, seed: int = 0, layer: int = 0, peaked: bool = False,
                layouts=None, n_q: Optional[int] = None,
                parent: Optional[np.ndarray] = "cfg") -> VerifyCase:
    """`peaked` scales Q by 4 so that scores have std ~4 and the softmax is
    dominated by a few keys (outputs of order 1 even at 26k context)."""
    layouts = layouts if layouts is not None else layouts_of(cfg, seed)
    B = len(layouts)
    n_q = cfg.n_q if n_q is None else n_q
    if isinstance(parent, str):
        parent = parent_of(cfg, seed) if n_q == cfg.n_q else None
    lens = [layout_length(l) + n_q for l in layouts]
    cu = np.concatenate(([0], np.cumsum(lens))).astype(np.int32)
    rng = _rng(seed, 201, layer)
    T = int(cu[-1])
    q = _normal(rng, (B * n_q, cfg.n_q_heads, cfg.head_dim), cfg.dtype, 4.0 if peaked else 1.0)
    k = _normal(rng, (T, cfg.n_kv_heads, cfg.head_dim), cfg.dtype)
    v = _normal(rng, (T, cfg.n_kv_heads, cfg.head_dim), cfg.dtype)
    return VerifyCase(cfg, q, k, v, cu, parent, n_q)


def lm_head_weights(cfg: Config, seed: int = 0, vocab: Optional[int] = None) -> np.ndarray:
    """[V, H] ~ N(0, std 0.02) (initialiser-range convention), storage-rounded.
    Drawn in row blocks so that the first `vocab` rows do not depend on V."""
    V = cfg.vocab if vocab is None else vocab
    out = np.empty((V, cfg.hidden), dtype=np.float32)
    blk = 8192

    def fill(i: int) -> None:
        r0 = i * blk
        r1 = min(V, r0 + blk)
        rng = _rng(seed, 501, i)
        out[r0:r1] = _normal(rng, (blk, cfg.hidden), cfg.dtype, 0.02)[: r1 - r0]

    n_blk = (V + blk - 1) // blk
    if n_blk == 1:
        fill(0)
    else:   # independent streams per block: drawing them concurrently changes nothing
        with ThreadPoolExecutor(max_workers=min(8, n_blk)) as pool:
            list(pool.map(fill, range(n_blk)))
    return out


def accept_case(cfg: Config, seed: int = 0, vocab: Optional[int] = None,
                batch: Optional[int] = None, n_q: Optional[int] = None,
                parent="cfg", lm_head: Optional[np.ndarray] = None,
                planted: bool = False) -> AcceptCase:
    """Random hidden rows ~ N(0,1) and uniformly random draft ids.  With
    `planted`, row r is instead a scaled copy of lm_head row planted_ids[r]
    plus small noise, so that this row's largest logit is at planted_ids[r]
    with a wide margin (Cauchy-Schwarz on near-equal-norm rows)."""
    B = cfg.batch if batch is None else batch
    n_q = cfg.n_q if n_q is None else n_q
    if isinstance(parent, str):
        parent = parent_of(cfg, seed) if n_q == cfg.n_q else None
    W = lm_head if lm_head is not None else lm_head_weights(cfg, seed, vocab)
    V = W.shape[0]
    rng = _rng(seed, 601)
    rows = B * (n_q + 1)
    planted_ids = None
    if planted:
        planted_ids = rng.integers(0, V, size=rows).astype(np.int32)
        noise = rng.standard_normal(size=(rows, cfg.hidden), dtype=np.float32) * np.float32(0.05)
        hidden = to_storage(W[planted_ids] * np.float32(50.0) + noise, cfg.dtype)
    else:
        hidden = _normal(rng, (rows, cfg.hidden), cfg.dtype)
    draft_ids = rng.integers(0, V, size=B * n_q).astype(np.int32)
    return AcceptCase(cfg, hidden, W, draft_ids, parent, n_q, planted_ids)


@dataclass
class HsrCase:
    """Inputs of the draft's input side for M new tokens (one per sequence in a
    chain draft): the embedding table and token ids, the target's hidden state
    of the previous step, the FC projection of the concatenation (Eq. 1), and
    the draft layer's input norm, QKV projection and rotary rows."""
    cfg: Config
    embed: np.ndarray        # [V, H]
    token_ids: np.ndarray    # int32 [M]
    h_prev: np.ndarray       # [M, H]
    w_fc: np.ndarray         # [H, 2H]
    b_fc: np.ndarray         # [H]
    norm_weight: np.ndarray  # [H]
    eps: float
    w_qkv: np.ndarray        # [(Hq + 2 Hkv) d, H]
    b_qkv: np.ndarray        # [(Hq + 2 Hkv) d]
    positions: np.ndarray    # int32 [M], sequence-local position of every new token
    rope_cos: np.ndarray     # float32 [M, d/2]
    rope_sin: np.ndarray     # float32 [M, d/2]


def rope_rows(positions: np.ndarray, head_dim: int, theta: float = 1.0e6):
    """float32 (cos, sin) [M, d/2] rows of a rotary table, angle = pos * theta^(-2i/d); the
    caller of the library owns this table (one per forward pass, shared by all layers)."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * theta ** (-2.0 * i / head_dim)[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def hsr_case(cfg: Config, seed: int = 0, rows: Optional[int] = None,
             embed: Optional[np.ndarray] = None, vocab: Optional[int] = None,
             positions: Optional[np.ndarray] = None) -> HsrCase:
    """Weights ~ N(0, 0.02) (initialiser range), biases N(0, 0.02) / N(0, 0.5) (QKV biases of
    the Qwen2 family are of order 1), norm weight 1 + N(0, 0.1), hidden state N(0, 1).  `embed`
    may be any [V, H] table (the benchmark passes the lm_head matrix it already holds)."""
    M = cfg.batch if rows is None else rows
    H, d = cfg.hidden, cfg.head_dim
    N = (cfg.n_q_heads + 2 * cfg.n_kv_heads) * d
    rng = _rng(seed, 701)
    if embed is None:
        embed = lm_head_weights(cfg, seed + 7919, vocab)
    V = embed.shape[0]
    token_ids = rng.integers(0, V, size=M).astype(np.int32)
    h_prev = _normal(rng, (M, H), cfg.dtype)
    w_fc = _normal(rng, (H, 2 * H), cfg.dtype, 0.02)
    b_fc = _normal(rng, (H,), cfg.dtype, 0.02)
    norm_weight = to_storage(1.0 + 0.1 * rng.standard_normal(size=H, dtype=np.float32), cfg.dtype)
    w_qkv = _normal(rng, (N, H), cfg.dtype, 0.02)
    b_qkv = _normal(rng, (N,), cfg.dtype, 0.5)
    if positions is None:
        lens = [layout_length(l) for l in layouts_of(cfg, seed)]
        positions = np.array([lens[m % len(lens)] - 1 + m // len(lens) for m in range(M)])
    positions = np.asarray(positions, dtype=np.int32)
    cs, sn = rope_rows(positions, d)
    return HsrCase(cfg, embed, token_ids, h_prev, w_fc, b_fc, norm_weight, 1e-6, w_qkv, b_qkv,
                   positions, cs, sn)
