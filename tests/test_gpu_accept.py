"""GPU parity: dream_accept_path against the oracle, bit-exact on every integer output."""
import numpy as np
import pytest

import dream_inputs as di
import oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from tests import gpu_util
    return gpu_util


def _compare(gu, logits, dtype, token, parent, max_depth):
    got = gu.run_accept(logits, dtype, token, parent, max_depth)
    want = oracle.accept_path(logits, dtype, token, parent, max_depth)
    for g, w, what in zip(got, want, ("node_argmax", "accept_len", "accept_path", "bonus_token")):
        assert np.array_equal(g, w), what
    return got


def test_tiny_config_every_plant_depth(gu):
    cfg = di.CONFIGS["tiny"]
    for d in range(cfg.depth + 1):
        logits, token, parent, ends = di.accept_inputs(cfg, plant_depths=[d])
        got = _compare(gu, logits, cfg.dtype, token, parent, cfg.depth)
        assert got[1][0] == d


@pytest.mark.parametrize("name", ["llava", "pixtral", "gemma3", "smolvlm_b8", "smolvlm_b32"])
def test_full_size_configs(gu, name):
    cfg = di.CONFIGS[name]
    logits, token, parent, ends = di.accept_inputs(cfg, n_ties=2)
    got = _compare(gu, logits, cfg.dtype, token, parent, cfg.depth)
    assert got[1].tolist() == [b % (cfg.depth + 1) for b in range(cfg.batch)]
    assert (got[1] + 1 <= 7).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("vocab", [1, 7, 1000, 8191, 8192, 8193, 32003])
def test_ragged_vocab_and_planted_ties(gu, dtype, vocab):
    T = 13
    parent = di.random_tree(T, 4, 5 + vocab)
    token = di.tree_tokens(parent, max(vocab, T), 6)[None] % vocab
    logits = di.normal((2, T, vocab), dtype, 70 + vocab, di.STREAM_LOGITS)
    top = np.float32(9.0) if dtype == "f32" else di.f32_to_bf16_bits(np.array([9.0], dtype=np.float32))[0]
    g = di.rng(3, 902, vocab)
    for b in range(2):
        for i in range(T):
            cols = g.integers(0, vocab, size=3)
            logits[b, i, cols] = top                      # exact ties at the maximum, anywhere in the row
    _compare(gu, logits, dtype, np.repeat(token, 2, 0), np.repeat(parent[None], 2, 0), 4)


def test_duplicate_siblings_chain_and_single_node(gu):
    parent = np.array([[-1, 0, 0, 1, 2]], dtype=np.int32)
    token = np.array([[0, 5, 5, 6, 6]], dtype=np.int32)
    logits = np.zeros((1, 5, 8), dtype=np.float32)
    logits[0, 0, 5] = 1
    logits[0, 1, 6] = 1
    logits[0, 2, 6] = 1
    logits[0, 3, 2] = 1
    got = _compare(gu, logits, "f32", token, parent, 4)
    assert got[2][0].tolist() == [0, 1, 3, -1, -1]
    # chain deeper than max_depth
    parent = di.chain_tree(9)[None]
    token = np.ones((1, 9), dtype=np.int32)
    logits = np.zeros((1, 9, 4), dtype=np.float32)
    logits[0, :, 1] = 1
    got = _compare(gu, logits, "f32", token, parent, 6)
    assert got[1][0] == 6
    got = _compare(gu, logits[:, :1], "f32", token[:, :1], parent[:, :1], 6)
    assert got[1][0] == 0


def test_large_tree_of_1024_nodes(gu):
    T = 1024
    parent = di.random_tree(T, 12, 77)
    token = di.tree_tokens(parent, 50, 78)
    logits = di.normal((1, T, 50), "bf16", 79, di.STREAM_LOGITS)
    _compare(gu, logits, "bf16", token[None], parent[None], 12)


def test_parent_array_with_cycles_still_terminates(gu):
    """Device metadata is trusted, but a malformed parent array must end in unspecified results, not in a hang."""
    T, V = 8, 16
    parent = np.array([[-1, 1, 3, 2, 9, 4, -5, 0]], dtype=np.int32)      # self loop, 2<->3 cycle, out of range, negative
    token = np.full((1, T), 3, dtype=np.int32)
    logits = np.zeros((1, T, V), dtype=np.float32)
    logits[0, :, 3] = 1                                                     # every edge "matches"
    am, alen, path, bonus = gu.run_accept(logits, "f32", token, parent, 6)
    assert (am == 3).all() and 0 <= alen[0] <= 6 and bonus[0] == 3
    assert ((path >= -1) & (path < T)).all()
    assert alen[0] == 1 and path[0].tolist()[:2] == [0, 7]                  # only node 7 has a well-formed path
