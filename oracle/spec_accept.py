"""Stochastic (temperature > 0) acceptance over a verified draft tree, float64 numpy.  TEST INFRASTRUCTURE ONLY.

What it follows: the acceptance rule of Section 2.1 -- a drafted token d is accepted with probability
min(1, P_target(d) / P_draft(d)); after a rejection everything later is discarded and the target's own
distribution decides the token that continues the sequence -- which the paper says is compatible with any
sampling temperature and evaluates at temperature 1 (Section 4, Table 1).  The paper states the rule for a chain
of drafts; for a tree (Section 3.1 drafts a tree) this build's reading is the usual multi-candidate form of the
same rule: at the current node its children are tried one after another in node order; after a rejected child the
target distribution becomes the normalised positive part of (target - draft), the rejected token is removed from
the draft distribution, and the next child is tried against those; the first accepted child becomes the current
node.  When no child is accepted (or the node has none) the token that continues the sequence is drawn from the
current (residual) target distribution by inverting its cumulative sum in token order.  The random numbers are
inputs: u_accept[b, i] for the test of node i, u_bonus[b] for the final draw.
Nothing here is shared with the HIP path."""
from __future__ import annotations

from typing import Tuple

import numpy as np


def _softmax(x: np.ndarray) -> np.ndarray:
    e = np.exp(x - x.max())
    return e / e.sum()


def spec_accept(target_logits_f64: np.ndarray, draft_logits_f64: np.ndarray, token: np.ndarray, parent: np.ndarray,
                u_accept: np.ndarray, u_bonus: np.ndarray, max_depth: int, inv_temperature: float = 1.0,
                flip_nodes=frozenset(), draw_window: float = 0.0):
    """logits [B,T,V] float64, token/parent [B,T], u_accept [B,T], u_bonus [B] ->
    (accept_len [B], accept_path [B,max_depth+1] (-1 padded), bonus_token [B], detail) where detail[b] lists, for
    diagnostics and gap guards, every acceptance test (node, ratio, u) and the final draw (target mass, cumulative
    sums around the drawn token).
    flip_nodes / draw_window do not belong to the method: they let a test enumerate what a lower-precision
    implementation may legitimately return when a comparison is too close to call.  The acceptance test of a node in
    flip_nodes takes the opposite outcome; detail[b]["draw_window_tokens"] lists every token of positive probability
    whose cumulative interval comes within draw_window (a fraction of the total mass) of the drawn point."""
    B, T, V = target_logits_f64.shape
    alen = np.zeros(B, dtype=np.int32)
    path = np.full((B, max_depth + 1), -1, dtype=np.int32)
    bonus = np.zeros(B, dtype=np.int32)
    detail = []
    for b in range(B):
        par = parent[b]
        children = [[] for _ in range(T)]
        for i in range(1, T):
            children[par[i]].append(i)
        cur, depth = 0, 0
        path[b, 0] = 0
        tests = []
        while True:
            p = _softmax(target_logits_f64[b, cur] * inv_temperature)
            kids = children[cur] if depth < max_depth else []
            accepted = -1
            if kids:
                q = _softmax(draft_logits_f64[b, cur] * inv_temperature)
                for c in kids:
                    x = int(token[b, c])
                    ratio = p[x] / q[x] if q[x] > 0 else (np.inf if p[x] > 0 else 0.0)
                    tests.append((c, float(ratio), float(u_accept[b, c])))
                    if (u_accept[b, c] < min(1.0, ratio)) != (c in flip_nodes):
                        accepted = c
                        break
                    r = np.maximum(p - q, 0.0)
                    if r.sum() > 0:
                        p = r / r.sum()
                    q = q.copy()
                    q[x] = 0.0
                    if q.sum() > 0:
                        q = q / q.sum()
            if accepted >= 0:
                cur = accepted
                depth += 1
                path[b, depth] = cur
                continue
            cdf = np.cumsum(p)
            target = u_bonus[b] * cdf[-1]
            t = int(np.searchsorted(cdf, target, side="right"))
            if t >= V:
                t = int(np.flatnonzero(p > 0)[-1])
            bonus[b] = t
            lo = cdf[t - 1] if t > 0 else 0.0
            w = draw_window * cdf[-1]
            first = int(np.searchsorted(cdf, target - w, side="left"))       # first token whose interval ends at or after target - w
            last = int(np.searchsorted(cdf, target + w, side="right"))       # last token whose interval starts at or before target + w
            near = [int(x) for x in range(max(first, 0), min(last, V - 1) + 1) if p[x] > 0]
            detail.append({"tests": tests, "draw_margin": float(min(target - lo, cdf[t] - target) / cdf[-1]), "draw_mass": float(p[t]),
                           "draw_window_tokens": near})
            break
        alen[b] = depth
    return alen, path, bonus, detail
