"""Pins of the oracle's draft-tree construction (Section 3.1: width-k expansion with top-k reordering as in
EAGLE-2; Section 4: k children, a depth, a budget of drafted tokens).  No GPU needed.

Closed forms (logits that are the logs of hand-chosen probabilities), invariances, hand-written rankings, and a
brute force over EVERY token sequence of a tiny vocabulary: whenever budget <= k the kept nodes must be exactly
the globally most probable prefixes (a node among the m <= k best overall has fewer than k better nodes on its
level and fewer than k better siblings, so the level-wise expansion cannot miss it)."""
import itertools

import numpy as np
import pytest

import dream_inputs as di
import oracle


def test_scores_are_the_log_probabilities_of_hand_chosen_distributions():
    p = np.array([[0.125, 0.5, 0.0625, 0.25, 0.0625], [0.2, 0.2, 0.2, 0.2, 0.2]])
    logits = np.log(p)[None] + np.array([[[3.0], [-7.0]]])          # a per-row shift must not matter
    cum = np.array([[-1.0, -2.5]])
    tok, score, nxt = oracle.expand_level(logits, cum, 3)
    assert tok[0, 0].tolist() == [1, 3, 0] and tok[0, 1].tolist() == [0, 1, 2]      # ties -> lower token
    np.testing.assert_allclose(score[0, 0], -1.0 + np.log([0.5, 0.25, 0.125]), atol=1e-13)
    np.testing.assert_allclose(score[0, 1], -2.5 + np.log([0.2, 0.2, 0.2]), atol=1e-13)
    # candidates flat: [0]: -1.69 [1]: -2.39 [2]: -3.08 [3..5]: -4.11 each -> frontier 0, 1, 2
    assert nxt[0].tolist() == [0, 1, 2]


def test_full_width_expansion_sums_to_one_and_uniform_rows():
    g = di.rng(1, 300)
    logits = g.normal(size=(2, 3, 11)) * 4
    cum = np.zeros((2, 3))
    tok, score, _ = oracle.expand_level(logits, cum, 11)
    np.testing.assert_allclose(np.exp(score).sum(axis=-1), 1.0, atol=1e-12)
    assert all(sorted(t.tolist()) == list(range(11)) for t in tok.reshape(-1, 11))
    assert (np.diff(score, axis=-1) <= 0).all()
    tok, score, nxt = oracle.expand_level(np.full((1, 2, 7), 2.5), np.array([[0.0, 0.0]]), 4)
    assert tok[0].tolist() == [[0, 1, 2, 3]] * 2
    np.testing.assert_allclose(score, -np.log(7.0), atol=1e-13)
    assert nxt[0].tolist() == [0, 1, 2, 3]                                           # all equal -> lowest flat indices


def test_frontier_ranking_written_out_by_hand():
    # two frontier nodes, k = 2: scores 0:-0.3 1:-2.0 | 2:-0.9 3:-0.9 -> order 0, 2, 3 (tie -> lower), 1
    logits = np.array([[[0.0, -1.7, -50.0], [5.0, 5.0, -50.0]]])
    lse0 = np.log(np.exp(logits[0, 0]).sum())
    lse1 = np.log(np.exp(logits[0, 1]).sum())
    cum = np.array([[-0.3 + lse0, -0.9 + lse1 - 5.0]])
    tok, score, nxt = oracle.expand_level(logits, cum, 2)
    np.testing.assert_allclose(score[0], [[-0.3, -2.0], [-0.9, -0.9]], atol=1e-12)
    assert nxt[0].tolist() == [0, 2]
    assert tok[0].tolist() == [[0, 1], [0, 1]]


def test_finalize_keeps_the_best_in_creation_order_and_reindexes_parents():
    #            0(root) 1     2     3     4     5     6
    score = np.array([[9.9, -0.2, -1.5, -0.9, -0.4, -3.0, -1.1]])
    parent = np.array([[-1, 0, 0, 0, 1, 2, 1]], dtype=np.int32)
    token = np.array([[70, 71, 72, 73, 74, 75, 76]], dtype=np.int32)
    T, par, tok, pidx = oracle.finalize_tree(score, parent, token, 4)
    assert T == 5
    assert pidx[0].tolist() == [0, 1, 3, 4, 6]                     # -0.2, -0.4, -0.9, -1.1 survive
    assert par[0].tolist() == [-1, 0, 0, 1, 1] and tok[0].tolist() == [70, 71, 73, 74, 76]
    T, par, tok, pidx = oracle.finalize_tree(score, parent, token, 100)
    assert T == 7 and pidx[0].tolist() == list(range(7)) and par[0].tolist() == parent[0].tolist()
    tie = np.array([[0.0, -1.0, -1.0, -1.0]])
    T, par, tok, pidx = oracle.finalize_tree(tie, np.array([[-1, 0, 0, 0]], dtype=np.int32), token[:, :4], 2)
    assert pidx[0].tolist() == [0, 1, 2]
    with pytest.raises(ValueError):                                # a child scoring above its parent is not a tree of paths
        oracle.finalize_tree(np.array([[0.0, -5.0, -1.0]]), np.array([[-1, 0, 1]], dtype=np.int32), token[:, :3], 1)


def _table_draft(V, seed):
    """A synthetic draft whose next-token logits depend on the last two tokens of the path (a fixed random table)."""
    table = di.rng(seed, 301).normal(size=(V + 1, V + 1, V)) * 1.5
    return lambda path: table[path[-2] if len(path) > 1 else V, path[-1]]


@pytest.mark.parametrize("V,k,depth,budget,seed", [(4, 3, 3, 3, 1), (5, 4, 3, 4, 2), (3, 3, 4, 2, 3), (6, 2, 3, 2, 4), (4, 4, 4, 4, 5)])
def test_small_budgets_recover_the_globally_most_probable_prefixes(V, k, depth, budget, seed):
    draft = _table_draft(V, seed)
    out = oracle.build_tree(draft, root_token=0, k=k, depth=depth, budget=budget)
    # brute force: every token sequence of length 1..depth after the root, its log-probability under the draft
    every = []
    for L in range(1, depth + 1):
        for seq in itertools.product(range(V), repeat=L):
            lp, path = 0.0, [0]
            for t in seq:
                x = draft(path)
                lp += x[t] - np.log(np.exp(x).sum())
                path.append(t)
            every.append((lp, seq))
    every.sort(key=lambda e: -e[0])
    want = sorted(e[1] for e in every[:budget])
    got = []
    for i in range(1, out["n_tree"]):
        seq, a = [], i
        while a > 0:
            seq.append(int(out["token"][a]))
            a = int(out["parent"][a])
        got.append(tuple(seq[::-1]))
    assert sorted(got) == want
    assert abs(every[budget - 1][0] - every[budget][0]) > 1e-9      # the brute-force cut is not a tie


def test_paper_shaped_tree_properties():
    # k = 4 children, depth 6, at most 32 drafted tokens (Section 4)
    V = 50
    draft = _table_draft(V, 9)
    out = oracle.build_tree(draft, root_token=7, k=4, depth=6, budget=32)
    assert out["pool_score"].shape[0] == 1 + 4 + 5 * 16 and out["n_tree"] == 33
    par, lvl = out["parent"], out["pool_level"][out["pool_index"]]
    assert par[0] == -1 and all(0 <= par[i] < i for i in range(1, 33))
    assert all(lvl[i] == lvl[par[i]] + 1 for i in range(1, 33)) and lvl.max() <= 6
    s = out["pool_score"][out["pool_index"]]
    assert all(s[i] <= s[par[i]] + 1e-12 for i in range(1, 33) if par[i] > 0)          # path probabilities only shrink
    dropped = np.setdiff1d(np.arange(1, 85), out["pool_index"])
    assert out["pool_score"][dropped].max() <= s[1:].min() + 1e-12                      # nothing better was dropped
    for i in range(1, 33):                                                              # siblings carry distinct tokens
        sib = [int(out["token"][j]) for j in range(1, 33) if par[j] == par[i]]
        assert len(sib) == len(set(sib))
