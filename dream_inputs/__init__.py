"""Seeded synthetic inputs for the DREAM decode-step hot path.

This module only *draws* inputs: random tensors, draft trees, drafted tokens and
logits with a planted accepted path.  It contains none of the method's
arithmetic (no attention, no scoring, no top-k, no acceptance), so both the CPU
oracle's tests and the HIP path's tests may import it without sharing any code
that computes a result.

Shapes follow the five measurement configurations (tiny / LLaVA-1.5-7B /
Pixtral-12B / Gemma3-12B / SmolVLM batch sweep); the tree shapes follow the
paper's Section 4 set-up (k = 4 children, depth 6, at most 32 drafted tokens)
and the 60-node, depth-6, root-top-10 tree the measurement configurations name.

bf16 tensors are carried as numpy uint16 arrays holding the raw bit patterns;
fp32 values are rounded to bf16 once (round-to-nearest-even) here, so every
consumer reads identical bytes.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 20250519

# stream ids: one independent random stream per tensor kind
STREAM_Q, STREAM_K, STREAM_V, STREAM_TREE, STREAM_TOKEN, STREAM_LOGITS = 1, 2, 3, 4, 5, 6
STREAM_XQ, STREAM_XK, STREAM_XV, STREAM_PREFILL_Q, STREAM_ROWS, STREAM_SCORES = 7, 8, 9, 10, 11, 12
STREAM_PLANT = 13
STREAM_DRAFT_LOGITS, STREAM_CUM = 14, 15


@dataclass(frozen=True)
class Config:
    """One measurement configuration (shapes only)."""
    name: str
    dtype: str            # "f32" or "bf16"
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    hidden: int
    n_visual: int         # v
    n_text: int           # q
    n_tree: int           # T, root included
    depth: int            # maximum node depth (root = 0)
    keep_num: int
    keep_den: int
    vocab: int
    n_layers: int         # harness parameter: target layers looped per decode step
    index: int            # position in the configuration list (seed offset)

    @property
    def prefix(self) -> int:
        return self.n_visual + self.n_text

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    def with_batch(self, batch: int) -> "Config":
        return replace(self, batch=batch, name=f"{self.name.split('_b')[0]}_b{batch}")


CONFIGS: Dict[str, Config] = {
    "tiny": Config("tiny", "f32", 1, 4, 4, 64, 256, 64, 32, 8, 3, 1, 2, 1000, 1, 0),
    "llava": Config("llava", "bf16", 1, 32, 32, 128, 4096, 576, 128, 60, 6, 1, 4, 32000, 32, 1),
    "pixtral": Config("pixtral", "bf16", 1, 32, 8, 128, 5120, 1024, 256, 60, 6, 1, 4, 131072, 40, 2),
    "gemma3": Config("gemma3", "bf16", 1, 16, 8, 256, 3840, 256, 1024, 60, 6, 1, 2, 262144, 48, 3),
    "smolvlm_b1": Config("smolvlm_b1", "bf16", 1, 32, 32, 64, 2048, 1088, 512, 60, 6, 1, 4, 49152, 24, 4),
}
CONFIGS["smolvlm_b8"] = CONFIGS["smolvlm_b1"].with_batch(8)
CONFIGS["smolvlm_b32"] = CONFIGS["smolvlm_b1"].with_batch(32)

LEVEL_SIZES_60 = (1, 10, 10, 10, 10, 10, 9)   # 60 nodes, depth 6, root top-10 branching


# --------------------------------------------------------------------------- #
# random streams and dtype plumbing
# --------------------------------------------------------------------------- #
def rng(seed: int, stream: int, sub: int = 0) -> np.random.Generator:
    """Counter-based generator: (seed, stream, sub) selects an independent Philox stream."""
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64((stream << 32) | sub)]))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal(shape: Sequence[int], dtype: str, seed: int, stream: int, sub: int = 0) -> np.ndarray:
    """N(0,1) tensor.  dtype "f32" -> float32 array, "bf16" -> uint16 bit patterns."""
    x = rng(seed, stream, sub).standard_normal(size=tuple(shape), dtype=np.float32)
    return x if dtype == "f32" else f32_to_bf16_bits(x)


def as_f64(x: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of a stored tensor to float64 (for building expectations in tests)."""
    return (x if dtype == "f32" else bf16_bits_to_f32(x)).astype(np.float64)


# --------------------------------------------------------------------------- #
# draft trees
# --------------------------------------------------------------------------- #
def tree_depths(parent: np.ndarray) -> np.ndarray:
    parent = np.asarray(parent)
    d = np.zeros(parent.shape[-1], dtype=np.int32)
    for i in range(1, parent.shape[-1]):
        d[i] = d[parent[i]] + 1
    return d


def level_tree(level_sizes: Sequence[int], seed: int, sub: int = 0) -> np.ndarray:
    """Level-ordered tree: node 0 is the root; every node of level l >= 1 picks a parent in
    level l-1 with probability proportional to 1/(rank+1) (confidence-ranked expansion puts
    more children under the better-ranked parents).  The first node of each level hangs off
    the first node of the level above, so the last level is always reached."""
    g = rng(seed, STREAM_TREE, sub)
    parent: List[int] = [-1]
    start_prev, start = 0, 1
    for lvl in range(1, len(level_sizes)):
        n_prev, n = level_sizes[lvl - 1], level_sizes[lvl]
        w = 1.0 / (np.arange(n_prev) + 1.0)
        picks = g.choice(n_prev, size=n, p=w / w.sum())
        picks[0] = 0
        picks.sort()                                   # keeps siblings contiguous
        parent.extend(int(start_prev + p) for p in picks)
        start_prev, start = start, start + n
    return np.asarray(parent, dtype=np.int32)


def random_tree(n_tree: int, max_depth: int, seed: int, sub: int = 0) -> np.ndarray:
    """parent[i] uniform in [0, i) subject to depth <= max_depth; one chain of depth max_depth
    is forced through nodes 1..max_depth."""
    g = rng(seed, STREAM_TREE, sub)
    parent = np.full(n_tree, -1, dtype=np.int32)
    depth = np.zeros(n_tree, dtype=np.int32)
    for i in range(1, n_tree):
        if i <= max_depth:
            p = i - 1
        else:
            while True:
                p = int(g.integers(0, i))
                if depth[p] < max_depth:
                    break
        parent[i] = p
        depth[i] = depth[p] + 1
    return parent


def kary_budget_tree(k: int = 4, depth: int = 6, budget: int = 32, seed: int = BASE_SEED, sub: int = 0) -> np.ndarray:
    """Paper-shaped tree (Section 4 set-up: k children per node, the given depth, at most
    `budget` drafted tokens, root excluded).  Level 1 has k nodes; the remaining budget is spread
    evenly over the deeper levels; parents are drawn like in level_tree, with no node receiving
    more than k children."""
    rest, lv = budget - k, depth - 1
    sizes = [1, k] + [rest // lv + (1 if i < rest % lv else 0) for i in range(lv)]
    g = rng(seed, STREAM_TREE, sub)
    parent: List[int] = [-1]
    start_prev, start = 0, 1
    for lvl in range(1, len(sizes)):
        n_prev, n = sizes[lvl - 1], sizes[lvl]
        assert n <= n_prev * k
        w = 1.0 / (np.arange(n_prev) + 1.0)
        picks = g.choice(n_prev, size=n, p=w / w.sum())
        picks[0] = 0
        counts = np.bincount(picks, minlength=n_prev)
        while counts.max() > k:                         # move surplus children to the emptiest parent
            counts[int(np.argmax(counts))] -= 1
            counts[int(np.argmin(counts))] += 1
        for p_idx, c in enumerate(counts):
            parent.extend([start_prev + p_idx] * int(c))
        start_prev, start = start, start + n
    return np.asarray(parent, dtype=np.int32)


def chain_tree(n_tree: int) -> np.ndarray:
    return np.arange(-1, n_tree - 1, dtype=np.int32)


def star_tree(n_tree: int) -> np.ndarray:
    p = np.zeros(n_tree, dtype=np.int32)
    p[0] = -1
    return p


def config_tree(cfg: Config, seq: int = 0) -> np.ndarray:
    """The tree of sequence `seq` for a configuration (tree seed = config seed, sub-stream = seq)."""
    if cfg.n_tree == sum(LEVEL_SIZES_60) and cfg.depth == len(LEVEL_SIZES_60) - 1:
        return level_tree(LEVEL_SIZES_60, cfg.seed, seq)
    return random_tree(cfg.n_tree, cfg.depth, cfg.seed, seq)


def ancestor_mask_bits(parent: np.ndarray, include_self: bool) -> np.ndarray:
    """Tree mask as bit words: word w of row i has bit (a % 64) set iff node a = 64*w + (a % 64)
    is visible to node i.  Pure tree bookkeeping for the optional explicit-mask argument."""
    parent = np.asarray(parent)
    n = parent.shape[-1]
    words = (n + 63) // 64
    out = np.zeros((n, words), dtype=np.uint64)
    for i in range(n):
        a = i if include_self else int(parent[i])
        while a >= 0:
            out[i, a // 64] |= np.uint64(1) << np.uint64(a % 64)
            a = int(parent[a])
    return out


# --------------------------------------------------------------------------- #
# drafted tokens and logits
# --------------------------------------------------------------------------- #
def tree_tokens(parent: np.ndarray, vocab: int, seed: int, sub: int = 0) -> np.ndarray:
    """One drafted token per node, siblings pairwise distinct (top-k expansion never repeats a
    token under one parent).  token[0] is the root's (already accepted) token."""
    g = rng(seed, STREAM_TOKEN, sub)
    parent = np.asarray(parent)
    n = parent.shape[0]
    token = np.zeros(n, dtype=np.int32)
    token[0] = int(g.integers(0, vocab))
    for p in range(n):
        kids = np.nonzero(parent == p)[0]
        if kids.size:
            token[kids] = g.choice(vocab, size=kids.size, replace=False).astype(np.int32)
    return token


def path_to(parent: np.ndarray, node: int) -> List[int]:
    out = []
    a = int(node)
    while a >= 0:
        out.append(a)
        a = int(parent[a])
    return out[::-1]


def accepted_paths(parents: np.ndarray, depths: Sequence[int], max_depth: int, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """For every sequence a root-to-node path to a seeded node at the asked depth, in the layout the
    acceptance step emits: path [B, max_depth+1] root first and -1 padded, accept_len [B]."""
    B = parents.shape[0]
    path = np.full((B, max_depth + 1), -1, dtype=np.int32)
    alen = np.zeros(B, dtype=np.int32)
    for b in range(B):
        node = node_at_depth(parents[b], int(depths[b]), seed, sub=b)
        p = path_to(parents[b], node)
        path[b, :len(p)] = p
        alen[b] = len(p) - 1
    return path, alen


def node_at_depth(parent: np.ndarray, depth: int, seed: int, sub: int = 0) -> int:
    d = tree_depths(parent)
    cand = np.nonzero(d == depth)[0]
    assert cand.size, "no node at that depth"
    return int(cand[int(rng(seed, STREAM_PLANT, sub).integers(0, cand.size))])


def planted_logits(parent: np.ndarray, token: np.ndarray, vocab: int, dtype: str, seed: int,
                   plant_depth: int, sub: int = 0, boost: float = 16.0,
                   n_ties: int = 0) -> Tuple[np.ndarray, int]:
    """N(0,1) logits [T, V] in `dtype`; along the path to a seeded node of depth `plant_depth`
    the entry logits[node, token[child]] is raised by `boost`, so the target's greedy choice
    follows that path.  At the path's end node (and at every node off the path) the greedy
    choice is left to the noise, except that it is steered away from that node's children so
    the planted depth is exact.  With n_ties > 0 the maximum of each row is duplicated
    exactly at n_ties further seeded columns above it (tie-break exercise).
    Returns (logits, end_node)."""
    parent = np.asarray(parent)
    n = parent.shape[0]
    g = rng(seed, STREAM_LOGITS, sub)
    x = g.standard_normal(size=(n, vocab), dtype=np.float32)
    end = node_at_depth(parent, plant_depth, seed, sub)
    path = path_to(parent, end)
    for a, c in zip(path[:-1], path[1:]):
        x[a, token[c]] += np.float32(boost)
    # off-path nodes and the end node: make sure the row maximum is not one of their children
    on_path_parent = set(path[:-1])
    for a in range(n):
        if a in on_path_parent:
            continue
        kids = np.nonzero(parent == a)[0]
        if kids.size:
            x[a, token[kids]] -= np.float32(boost)
    if dtype == "bf16":
        xb = f32_to_bf16_bits(x)
        xv = bf16_bits_to_f32(xb)
    else:
        xb, xv = x, x
    if n_ties > 0:
        gt = rng(seed, STREAM_LOGITS, sub + 7919)
        for a in range(n):
            j = int(np.argmax(xv[a]))
            later = np.arange(j + 1, vocab)
            if later.size == 0:
                continue
            cols = gt.choice(later, size=min(n_ties, later.size), replace=False)
            xb[a, cols] = xb[a, j]
    return xb, end


# --------------------------------------------------------------------------- #
# attention inputs
# --------------------------------------------------------------------------- #
@dataclass
class AttnInputs:
    q: np.ndarray            # [B, Tq, Hq, D]
    k: np.ndarray            # [B, Hkv, s_max, D]
    v: np.ndarray            # [B, Hkv, s_max, D]
    prefix_len: np.ndarray   # [B] int32
    parent: np.ndarray       # [B, T] int32
    s_max: int
    dtype: str


def _poison(dtype: str) -> np.ndarray:
    big = np.float32(3.0e4)
    return big if dtype == "f32" else f32_to_bf16_bits(np.array([big]))[0]


def verify_inputs(cfg: Config, seed: Optional[int] = None, prefix_len: Optional[Sequence[int]] = None,
                  parents: Optional[np.ndarray] = None, slack_rows: int = 5,
                  streams: Tuple[int, int, int] = (STREAM_Q, STREAM_K, STREAM_V), sub: int = 0) -> AttnInputs:
    """Q for the T tree nodes and a K/V cache whose rows [0, P) are the prefix and [P, P+T) the
    tree nodes' own K/V.  Rows at and beyond P+T (cache slack) hold a huge value, so a kernel that
    reads past the live rows fails parity loudly."""
    seed = cfg.seed if seed is None else seed
    B, T, D = cfg.batch, cfg.n_tree, cfg.head_dim
    pl = np.full(B, cfg.prefix, dtype=np.int32) if prefix_len is None else np.asarray(prefix_len, dtype=np.int32)
    s_max = int(pl.max()) + T + slack_rows
    q = normal((B, T, cfg.n_q_heads, D), cfg.dtype, seed, streams[0], sub)
    k = normal((B, cfg.n_kv_heads, s_max, D), cfg.dtype, seed, streams[1], sub)
    v = normal((B, cfg.n_kv_heads, s_max, D), cfg.dtype, seed, streams[2], sub)
    for b in range(B):
        k[b, :, pl[b] + T:, :] = _poison(cfg.dtype)
        v[b, :, pl[b] + T:, :] = _poison(cfg.dtype)
    if parents is None:
        parents = np.stack([config_tree(cfg, b) for b in range(B)])
    return AttnInputs(q, k, v, pl, np.ascontiguousarray(parents, dtype=np.int32), s_max, cfg.dtype)


def tree_levels(parent: np.ndarray) -> List[np.ndarray]:
    d = tree_depths(parent)
    return [np.nonzero(d == l)[0].astype(np.int32) for l in range(int(d.max()) + 1)]


def xattn_inputs(cfg: Config, seed: Optional[int] = None, slack_rows: int = 5) -> AttnInputs:
    """Draft cross-attention operands: K/V rows [0, n) stand for the projected target features,
    rows [n, n+T) for the projected draft features of the tree nodes; Q holds one row per tree
    node (callers pass the rows of one tree level per call)."""
    return verify_inputs(cfg, seed, slack_rows=slack_rows, streams=(STREAM_XQ, STREAM_XK, STREAM_XV))


def prefill_q(cfg: Config, n_q: Optional[int] = None, seed: Optional[int] = None) -> np.ndarray:
    """Last-layer queries of the prefill rows, [B, n_q, Hq, D] (row r sits at position r)."""
    n_q = cfg.prefix if n_q is None else n_q
    seed = cfg.seed if seed is None else seed
    return normal((cfg.batch, n_q, cfg.n_q_heads, cfg.head_dim), cfg.dtype, seed, STREAM_PREFILL_Q)


def feature_rows(cfg: Config, n_rows: Optional[int] = None, seed: Optional[int] = None) -> np.ndarray:
    """[B, P, hidden] token/feature matrix that the kept indices subsample."""
    n_rows = cfg.prefix if n_rows is None else n_rows
    seed = cfg.seed if seed is None else seed
    return normal((cfg.batch, n_rows, cfg.hidden), cfg.dtype, seed, STREAM_ROWS)


def accept_inputs(cfg: Config, plant_depths: Optional[Sequence[int]] = None, seed: Optional[int] = None,
                  parents: Optional[np.ndarray] = None, n_ties: int = 0):
    """(logits [B,T,V], token [B,T], parent [B,T], end_nodes [B]) with a planted accepted path per
    sequence; plant depth of sequence b defaults to b mod (depth+1)."""
    seed = cfg.seed if seed is None else seed
    B = cfg.batch
    if parents is None:
        parents = np.stack([config_tree(cfg, b) for b in range(B)])
    logits, tokens, ends = [], [], []
    for b in range(B):
        tok = tree_tokens(parents[b], cfg.vocab, seed, b)
        d = (b % (cfg.depth + 1)) if plant_depths is None else int(plant_depths[b])
        lg, end = planted_logits(parents[b], tok, cfg.vocab, cfg.dtype, seed, d, b, n_ties=n_ties)
        logits.append(lg)
        tokens.append(tok)
        ends.append(end)
    return (np.stack(logits), np.stack(tokens).astype(np.int32),
            np.ascontiguousarray(parents, dtype=np.int32), np.asarray(ends, dtype=np.int32))


def draft_level_inputs(batch: int, n_frontier: int, vocab: int, dtype: str, seed: int, level: int = 0,
                       spread: float = 3.0) -> Tuple[np.ndarray, np.ndarray]:
    """Draft logits [B,F,V] (N(0, spread^2), rounded once to `dtype`) of the frontier nodes of one tree level
    and their cumulative scores [B,F] float32 (negative, decreasing along the frontier as after a ranking)."""
    logits = normal((batch, n_frontier, vocab), "f32", seed, STREAM_DRAFT_LOGITS, level) * np.float32(spread)
    if dtype == "bf16":
        logits = f32_to_bf16_bits(logits)
    g = rng(seed, STREAM_CUM, level)
    cum = -np.sort(g.uniform(0.0, 3.0 * (level + 1), size=(batch, n_frontier)), axis=1).astype(np.float32)
    if level == 0:
        cum[:] = 0.0
    return logits, np.ascontiguousarray(cum)
