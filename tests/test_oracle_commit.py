"""Pins of the oracle's KV-cache commit (Section 2.1: after a rejection everything later is discarded and
decoding continues from the accepted prefix; Section 4: KV caching).  No GPU needed.

None of these re-types the oracle's copy loop: they use hand-written row markers, invariants of the
operation, and the meaning of the committed cache (attending to it must equal the tree-masked attention
of the accepted node, computed by the attention oracle on the ORIGINAL cache)."""
import numpy as np
import pytest

import dream_inputs as di
import oracle


def _marker_cache(B, Hkv, s_max, D):
    """float32 cache whose every element is 1000*b + 100*h + row: a row's identity is readable."""
    c = np.zeros((B, Hkv, s_max, D), dtype=np.float32)
    for b in range(B):
        for h in range(Hkv):
            c[b, h] = (1000 * b + 100 * h + np.arange(s_max, dtype=np.float32))[:, None]
    return c


def test_hand_written_markers_with_overlapping_moves():
    # prefix 3, tree rows 3..8 hold nodes 0..5; path root -> 2 -> 3 -> 5: the destination of the second move
    # (row 3+2) is the source of the first (node 2), so an in-place, in-order implementation would be wrong
    # the other way round; expected rows written out by hand
    c = _marker_cache(1, 2, 12, 4)
    out, new_len = oracle.kv_commit(c, "f32", [3], 6, [[0, 2, 3, 5, -1, -1, -1]], [3])
    assert new_len.tolist() == [7]
    for h in range(2):
        rows = out[0, h, :, 0] - 100 * h
        assert rows.tolist() == [0, 1, 2,       # prefix untouched
                                 3, 5, 6, 8,    # root (node 0), node 2, node 3, node 5
                                 7, 8,          # rest of the old tree area keeps its old content
                                 9, 10, 11]     # rows behind the tree untouched
    assert np.all(out == out[..., :1])          # whole rows moved, not parts of them


def test_chain_path_is_a_no_op_and_commit_is_idempotent():
    cfg = di.CONFIGS["tiny"]
    inp = di.verify_inputs(cfg, parents=np.stack([di.chain_tree(cfg.n_tree)]))
    d = 5
    path = np.full((1, cfg.n_tree), -1, dtype=np.int32)
    path[0, :d + 1] = np.arange(d + 1)
    out, new_len = oracle.kv_commit(inp.k, inp.dtype, inp.prefix_len, cfg.n_tree, path, [d])
    assert np.array_equal(out.view(np.uint32), inp.k.view(np.uint32))
    assert new_len.tolist() == [int(inp.prefix_len[0]) + d + 1]
    # the committed rows form a chain again: committing the chain path a second time changes nothing
    out2, _ = oracle.kv_commit(out, inp.dtype, inp.prefix_len, cfg.n_tree, path, [d])
    assert np.array_equal(out2.view(np.uint32), out.view(np.uint32))


@pytest.mark.parametrize("depth", [0, 1, 3])
def test_only_the_accepted_rows_move_and_other_sequences_are_untouched(depth):
    cfg = di.Config("c", "bf16", 3, 4, 2, 64, 256, 40, 13, 20, 4, 1, 2, 500, 1, 7)
    inp = di.verify_inputs(cfg, prefix_len=[53, 20, 41])
    path, alen = di.accepted_paths(inp.parent, [depth, 0, min(depth + 1, 4)], cfg.depth, cfg.seed)
    out, new_len = oracle.kv_commit(inp.k, "bf16", inp.prefix_len, cfg.n_tree, path, alen)
    assert new_len.tolist() == (inp.prefix_len + alen + 1).tolist()
    for b in range(cfg.batch):
        P, n = int(inp.prefix_len[b]), int(alen[b])
        assert np.array_equal(out[b, :, :P], inp.k[b, :, :P])                    # prefix
        assert np.array_equal(out[b, :, P + n + 1:], inp.k[b, :, P + n + 1:])    # everything behind the new end
        assert np.array_equal(out[b, :, P], inp.k[b, :, P])                      # the root never moves
        # the multiset of committed rows is the multiset of the path's rows (sorted by bit pattern)
        got = np.sort(out[b, :, P:P + n + 1].reshape(cfg.n_kv_heads, -1, cfg.head_dim), axis=1)
        want = np.sort(inp.k[b][:, P + path[b, :n + 1]], axis=1)
        assert np.array_equal(got, want)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_attending_to_the_committed_cache_equals_the_tree_masked_row_of_the_accepted_node(dtype):
    """The accepted node's visible set in verification is prefix + its root path (Section 3.1, tree mask).
    After the commit those are exactly rows [0, P+len+1) of the cache, so plain attention of that node's query
    over the committed cache (a one-node 'tree' whose prefix is P+len) must reproduce the tree-masked output.
    A commit that moved a wrong row, mixed heads up or mis-counted the new length changes this number."""
    cfg = di.Config("c", dtype, 2, 4, 2, 64, 256, 30, 7, 24, 5, 1, 2, 500, 1, 8)
    inp = di.verify_inputs(cfg, prefix_len=[37, 12])
    path, alen = di.accepted_paths(inp.parent, [4, 2], cfg.depth, cfg.seed)
    tree_out, _ = oracle.tree_attn(inp.q, inp.k, inp.v, dtype, inp.prefix_len, inp.parent, include_self=True)
    kc, new_len = oracle.kv_commit(inp.k, dtype, inp.prefix_len, cfg.n_tree, path, alen)
    vc, _ = oracle.kv_commit(inp.v, dtype, inp.prefix_len, cfg.n_tree, path, alen)
    best = np.array([path[b, alen[b]] for b in range(cfg.batch)])
    q1 = np.ascontiguousarray(np.stack([inp.q[b, best[b]] for b in range(cfg.batch)])[:, None])   # [B,1,Hq,D]
    single = np.full((cfg.batch, 1), -1, dtype=np.int32)
    flat_out, _ = oracle.tree_attn(q1, kc, vc, dtype, new_len - 1, single, include_self=True)
    for b in range(cfg.batch):
        np.testing.assert_allclose(flat_out[b, 0], tree_out[b, best[b]], rtol=0, atol=1e-12)


def test_out_of_range_paths_are_rejected_and_leave_no_result():
    c = _marker_cache(1, 1, 10, 2)
    with pytest.raises(ValueError):
        oracle.kv_commit(c, "f32", [2], 4, [[0, 4, -1]], [1])        # node 4 does not exist in a 4-node tree
    with pytest.raises(ValueError):
        oracle.kv_commit(c, "f32", [2], 4, [[0, 1, 2]], [3])         # length does not fit the path array
    with pytest.raises(ValueError):
        oracle.kv_commit(c, "f32", [8], 4, [[0, 1, 2]], [1])         # tree rows would not fit the cache
