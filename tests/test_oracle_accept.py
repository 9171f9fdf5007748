"""Pins for the oracle's per-node arg-max and greedy accepted path (Section 2.1 at temperature 0,
Section 4: one bonus token, at most depth + 1 tokens per round)."""
import os

import numpy as np
import pytest

import dream_inputs as di
import oracle


def _leaf_paths(parent):
    T = len(parent)
    leaves = [i for i in range(T) if not (np.asarray(parent) == i).any()]
    return [di.path_to(parent, l) for l in leaves]


def _brute_force(logits_f64, token, parent):
    """Enumerate every root-to-leaf path; walk it while the drafted token equals the arg-max at
    the previous node; the longest accepted prefix wins (first such path on ties)."""
    am = [int(np.flatnonzero(row == row.max())[0]) for row in logits_f64]
    best = [0]
    for path in _leaf_paths(parent):
        acc = [path[0]]
        for a, c in zip(path[:-1], path[1:]):
            if token[c] != am[a]:
                break
            acc.append(c)
        if len(acc) > len(best):
            best = acc
    return am, best


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_matches_root_to_leaf_enumeration(dtype):
    g = di.rng(8, 200)
    seen = set()
    for trial in range(300):
        T = int(g.integers(1, 14))
        V = int(g.integers(13, 16))                  # tiny vocab -> accepted paths of several lengths occur
        parent = di.random_tree(T, 5, 100 + trial) if T > 1 else np.array([-1], dtype=np.int32)
        token = di.tree_tokens(parent, V, 300 + trial) if T > 1 else np.array([0], dtype=np.int32)
        logits = di.normal((1, T, V), dtype, 400 + trial, di.STREAM_LOGITS)
        am, alen, path, bonus = oracle.accept_path(logits, dtype, token[None], parent[None], 6)
        want_am, want_path = _brute_force(di.as_f64(logits[0], dtype), token, parent)
        assert am[0].tolist() == want_am
        assert alen[0] == len(want_path) - 1
        assert path[0].tolist() == want_path + [-1] * (7 - len(want_path))
        assert bonus[0] == want_am[want_path[-1]]
        seen.add(int(alen[0]))
    assert {0, 1, 2} <= seen


def test_planted_paths_of_every_depth():
    cfg = di.CONFIGS["llava"]
    for d in range(cfg.depth + 1):
        logits, token, parent, ends = di.accept_inputs(cfg, plant_depths=[d], seed=cfg.seed + d)
        am, alen, path, bonus = oracle.accept_path(logits, "bf16", token, parent, cfg.depth)
        assert alen[0] == d
        want = di.path_to(parent[0], ends[0])
        assert path[0].tolist() == want + [-1] * (cfg.depth + 1 - len(want))
        assert bonus[0] == am[0, ends[0]]
        for a, c in zip(want[:-1], want[1:]):
            assert am[0, a] == token[0, c]
        assert alen[0] + 1 <= 7                                        # Section 4: up to 7 tokens a round


def test_root_argmax_matching_no_child_accepts_nothing():
    parent = di.star_tree(5)[None]
    token = np.array([[9, 1, 2, 3, 4]], dtype=np.int32)
    logits = np.zeros((1, 5, 10), dtype=np.float32)
    logits[0, 0, 7] = 1.0
    am, alen, path, bonus = oracle.accept_path(logits, "f32", token, parent, 3)
    assert alen[0] == 0 and path[0].tolist() == [0, -1, -1, -1] and bonus[0] == 7


def test_exact_bf16_ties_resolve_to_the_lowest_index():
    V = 4096
    x = di.normal((1, 3, V), "bf16", 77, di.STREAM_LOGITS)
    top = di.f32_to_bf16_bits(np.array([7.5], dtype=np.float32))[0]
    x[0, 0, [4000, 123, 2048]] = top
    x[0, 1, [V - 1, V - 2]] = top
    x[0, 2, 0] = top
    parent = np.array([[-1, 0, 1]], dtype=np.int32)
    token = np.array([[0, 123, V - 2]], dtype=np.int32)
    am, alen, path, bonus = oracle.accept_path(x, "bf16", token, parent, 2)
    assert am[0].tolist() == [123, V - 2, 0] and alen[0] == 2 and bonus[0] == 0
    # the generator's planted ties also keep the first maximum
    cfg = di.CONFIGS["tiny"]
    lg, tok, par, ends = di.accept_inputs(cfg, plant_depths=[2], n_ties=3)
    lg0, _, _, _ = di.accept_inputs(cfg, plant_depths=[2], n_ties=0)
    a1 = oracle.accept_path(lg, "f32", tok, par, cfg.depth)
    a0 = oracle.accept_path(lg0, "f32", tok, par, cfg.depth)
    assert not np.array_equal(lg, lg0)
    for u, w in zip(a1, a0):
        assert np.array_equal(u, w)


def test_duplicate_sibling_tokens_pick_the_lowest_node():
    parent = np.array([[-1, 0, 0, 1, 2]], dtype=np.int32)
    token = np.array([[0, 5, 5, 6, 6]], dtype=np.int32)
    logits = np.zeros((1, 5, 8), dtype=np.float32)
    logits[0, 0, 5] = 1
    logits[0, 1, 6] = 1
    logits[0, 2, 6] = 1
    logits[0, 3, 2] = 1
    am, alen, path, bonus = oracle.accept_path(logits, "f32", token, parent, 4)
    assert alen[0] == 2 and path[0].tolist() == [0, 1, 3, -1, -1] and bonus[0] == 2


def test_invariants_on_the_measurement_configs():
    for name in ("tiny", "llava", "smolvlm_b8"):
        cfg = di.CONFIGS[name]
        small = di.Config(cfg.name, cfg.dtype, cfg.batch, 1, 1, 8, 8, 1, 1, cfg.n_tree, cfg.depth, 1, 2, 2048, 1, cfg.index)
        logits, token, parent, ends = di.accept_inputs(small)
        am, alen, path, bonus = oracle.accept_path(logits, small.dtype, token, parent, cfg.depth)
        for b in range(cfg.batch):
            assert alen[b] == b % (cfg.depth + 1) <= cfg.depth
            nodes = [n for n in path[b] if n >= 0]
            assert nodes[0] == 0 and len(nodes) == alen[b] + 1
            assert all(parent[b, c] == a for a, c in zip(nodes[:-1], nodes[1:]))


def test_nodes_deeper_than_max_depth_are_ignored():
    parent = di.chain_tree(5)[None]
    token = np.array([[0, 1, 1, 1, 1]], dtype=np.int32)
    logits = np.zeros((1, 5, 4), dtype=np.float32)
    logits[0, :, 1] = 1
    am, alen, path, bonus = oracle.accept_path(logits, "f32", token, parent, 2)
    assert alen[0] == 2 and path[0].tolist() == [0, 1, 2]
