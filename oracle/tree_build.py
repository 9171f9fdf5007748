"""Draft-tree construction, float64 numpy.  TEST INFRASTRUCTURE ONLY (part of the oracle package).

What it follows: Section 3.1 (last paragraph) adopts the top-k reordering and tree expansion of EAGLE-2:
a width-k expansion of the drafted tree level by level, candidates ranked by the probability of their whole
path, and Section 4 fixes the shape (k children per node, a depth, a maximum number of drafted tokens).
The paper defers the details to supplementary material that is not available, so the steps below are this
build's reading of that published procedure, written in the order it is run:

  expand_level   for every frontier node: log-softmax of its draft logits; its k most probable tokens become
                 candidate children with score = score(node) + log p(token | node); the k best candidates of
                 the level (by score) form the next frontier.
  finalize_tree  after the last level: the root and the `budget` best candidates of all levels (by score) are
                 kept, listed in creation order (so a parent precedes its children), parents re-indexed.

Ties are resolved toward the lower token index / lower candidate index everywhere.  Token ranking inside a
row compares the logits themselves (the log-softmax is monotone), so it is exact for any input precision.
Nothing here is shared with the HIP path.
"""
from __future__ import annotations

from typing import Tuple

import numpy as np


def _rank_desc(values: np.ndarray) -> np.ndarray:
    """Indices sorted by (value descending, index ascending)."""
    idx = np.arange(values.shape[0])
    return np.lexsort((idx, -values))


def expand_level(logits_f64: np.ndarray, cum: np.ndarray, k: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """logits [B,F,V] (already widened to float64), cum [B,F] -> (cand_token [B,F,k] int32,
    cand_score [B,F,k] float64, next_frontier [B,min(k,F*k)] int32 flat indices f*k+j in rank order)."""
    B, F, V = logits_f64.shape
    assert 1 <= k <= V
    tok = np.zeros((B, F, k), dtype=np.int32)
    score = np.zeros((B, F, k), dtype=np.float64)
    kf = min(k, F * k)
    nxt = np.zeros((B, kf), dtype=np.int32)
    for b in range(B):
        for f in range(F):
            x = logits_f64[b, f]
            m = x.max()
            lse = m + np.log(np.exp(x - m).sum())
            order = _rank_desc(x)[:k]
            tok[b, f] = order
            score[b, f] = cum[b, f] + (x[order] - lse)
        nxt[b] = _rank_desc(score[b].reshape(-1))[:kf]
    return tok, score, nxt


def finalize_tree(pool_score: np.ndarray, pool_parent: np.ndarray, pool_token: np.ndarray, budget: int):
    """pool_* [B,N]: entry 0 is the root (its score is ignored), entry i > 0 has parent pool_parent[b,i] < i.
    Returns (n_tree, parent [B,T], token [B,T], pool_index [B,T]) with T = 1 + min(budget, N-1)."""
    B, N = pool_score.shape
    keep_n = min(budget, N - 1)
    T = 1 + keep_n
    parent = np.zeros((B, T), dtype=np.int32)
    token = np.zeros((B, T), dtype=np.int32)
    pidx = np.zeros((B, T), dtype=np.int32)
    for b in range(B):
        best = _rank_desc(np.asarray(pool_score[b, 1:], dtype=np.float64))[:keep_n] + 1
        kept = np.sort(np.concatenate([[0], best]))
        new_index = {int(p): i for i, p in enumerate(kept)}
        for i, p in enumerate(kept):
            pidx[b, i] = p
            token[b, i] = pool_token[b, p]
            if p == 0:
                parent[b, i] = -1
            else:
                pp = int(pool_parent[b, p])
                if pp not in new_index:
                    raise ValueError("kept candidate %d has a dropped parent %d: scores must not increase along a path" % (p, pp))
                parent[b, i] = new_index[pp]
    return T, parent, token, pidx


def build_tree(draft_logits, root_token: int, k: int, depth: int, budget: int):
    """Runs the whole procedure for ONE sequence with a caller-supplied draft: draft_logits(path_tokens) ->
    float64 logits [V] of the next token after the token path (root first).  Returns the pool
    (score, parent, token, level arrays) and the finalized tree."""
    pool_score, pool_parent, pool_token, pool_level = [0.0], [-1], [int(root_token)], [0]
    frontier = [0]
    frontier_gap = np.inf   # smallest distance between a score that made a frontier and the best one that did not
    for level in range(depth):
        paths = []
        for f in frontier:
            p, a = [], f
            while a >= 0:
                p.append(pool_token[a])
                a = pool_parent[a]
            paths.append(p[::-1])
        logits = np.stack([np.asarray(draft_logits(p), dtype=np.float64) for p in paths])[None]
        cum = np.asarray([[pool_score[f] for f in frontier]], dtype=np.float64)
        tok, score, nxt = expand_level(logits, cum, k)
        base = len(pool_score)
        for fi, f in enumerate(frontier):
            for j in range(k):
                pool_score.append(float(score[0, fi, j]))
                pool_parent.append(f)
                pool_token.append(int(tok[0, fi, j]))
                pool_level.append(level + 1)
        ranked = np.sort(score[0].reshape(-1))[::-1]
        if ranked.shape[0] > len(nxt[0]):
            frontier_gap = min(frontier_gap, float(ranked[len(nxt[0]) - 1] - ranked[len(nxt[0])]))
        frontier = [base + int(i) for i in nxt[0]]
    ps, pp, pt = (np.asarray(pool_score)[None], np.asarray(pool_parent, dtype=np.int32)[None],
                  np.asarray(pool_token, dtype=np.int32)[None])
    T, parent, token, pidx = finalize_tree(ps, pp, pt, budget)
    return {"pool_score": ps[0], "pool_parent": pp[0], "pool_token": pt[0], "pool_level": np.asarray(pool_level),
            "n_tree": T, "parent": parent[0], "token": token[0], "pool_index": pidx[0], "frontier_gap": frontier_gap}
