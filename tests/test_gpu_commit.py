"""GPU parity: dream_kv_commit against the oracle, bit for bit on every cache byte and on the new lengths."""
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


def _bits(a, dtype):
    return a.view(np.int32) if dtype == "f32" else a.view(np.int16)


def _compare(gu, caches, dtype, prefix_len, n_tree, path, alen):
    got, got_len = gu.run_commit(caches, dtype, prefix_len, n_tree, path, alen)
    for i, c in enumerate(caches):
        want, want_len = oracle.kv_commit(c, dtype, prefix_len, n_tree, path, alen)
        assert np.array_equal(got[i], _bits(want, dtype)), "cache %d differs" % i
        assert np.array_equal(got_len, want_len)


@pytest.mark.parametrize("name", ["tiny", "llava", "pixtral", "gemma3", "smolvlm_b8"])
def test_config_shapes_k_and_v_every_accept_depth(gu, name):
    cfg = di.CONFIGS[name]
    inp = di.verify_inputs(cfg)
    for d in range(cfg.depth + 1):
        depths = [(d + b) % (cfg.depth + 1) for b in range(cfg.batch)]
        path, alen = di.accepted_paths(inp.parent, depths, cfg.depth, cfg.seed + d)
        _compare(gu, [inp.k, inp.v], cfg.dtype, inp.prefix_len, cfg.n_tree, path, alen)


def test_overlapping_moves_and_chain(gu):
    # path 0,2,3,5: row 2 of the tree area is written by entry 2 and read by entry 1
    cfg = di.Config("c", "bf16", 2, 4, 2, 128, 512, 20, 9, 8, 7, 1, 2, 100, 1, 9)
    parents = np.stack([np.array([-1, 0, 0, 2, 2, 3, 5, 6], dtype=np.int32), di.chain_tree(8)])
    inp = di.verify_inputs(cfg, prefix_len=[29, 3], parents=parents)
    path = np.array([[0, 2, 3, 5, 6, 7, -1, -1], [0, 1, 2, 3, 4, 5, 6, 7]], dtype=np.int32)
    _compare(gu, [inp.k, inp.v], "bf16", inp.prefix_len, 8, path, [5, 7])
    _compare(gu, [inp.k], "bf16", inp.prefix_len, 8, path, [0, 0])


def test_more_caches_than_one_launch_carries(gu):
    cfg = di.Config("c", "f32", 1, 2, 2, 64, 128, 6, 2, 6, 3, 1, 2, 100, 1, 10)
    caches = [di.verify_inputs(cfg, sub=i).k for i in range(131)]
    inp = di.verify_inputs(cfg)
    path, alen = di.accepted_paths(inp.parent, [3], cfg.depth, cfg.seed)
    _compare(gu, caches, "f32", inp.prefix_len, cfg.n_tree, path, alen)


def test_accept_then_commit_then_attend(gu):
    """The round's tail as a caller runs it: dream_accept_path writes the path on the device, dream_kv_commit
    consumes it, and verification attention of the accepted node's query over the committed cache (a one-node
    tree behind the new prefix) equals the tree-masked row the oracle computes on the original cache."""
    import torch
    import paper_2505_19201_amd as dream
    cfg = di.CONFIGS["llava"]
    inp = di.verify_inputs(cfg)
    logits, token, parent, ends = di.accept_inputs(cfg, plant_depths=[4])
    assert np.array_equal(parent, inp.parent)
    B, T = cfg.batch, cfg.n_tree
    d_logits, d_token, d_parent = dream.to_device(logits, "bf16"), dream.to_device(token), dream.to_device(parent)
    am = torch.empty(B, T, dtype=torch.int32, device="cuda")
    alen = torch.empty(B, dtype=torch.int32, device="cuda")
    path = torch.empty(B, cfg.depth + 1, dtype=torch.int32, device="cuda")
    bonus = torch.empty(B, dtype=torch.int32, device="cuda")
    ws = dream.alloc_workspace(dream.dream_accept_path_workspace(B, T, cfg.vocab))
    dream.dream_accept_path(d_logits, dream.BF16, B, T, cfg.vocab, d_token, d_parent, cfg.depth, am, alen, path, bonus, ws)
    desc = dream.attn_desc(B, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, dream.BF16, inp.s_max)
    k, v = dream.to_device(inp.k, "bf16"), dream.to_device(inp.v, "bf16")
    pl = dream.to_device(inp.prefix_len)
    new_len = torch.empty(B, dtype=torch.int32, device="cuda")
    dream.dream_kv_commit(desc, [k, v], pl, T, path, alen, new_len)
    torch.cuda.synchronize()
    assert alen.cpu().tolist() == [4] and new_len.cpu().tolist() == [int(inp.prefix_len[0]) + 5]
    best = int(path.cpu().numpy()[0, 4])
    q1 = dream.to_device(np.ascontiguousarray(inp.q[:, best:best + 1]), "bf16")
    out = torch.empty(B, 1, cfg.n_q_heads, cfg.head_dim, dtype=torch.bfloat16, device="cuda")
    one = dream.to_device(np.full((B, 1), -1, dtype=np.int32))
    kv_len = int(new_len.max().item())
    ws2 = dream.alloc_workspace(dream.dream_tree_verify_attn_workspace(desc, 1, kv_len))
    dream.dream_tree_verify_attn(desc, q1, k, v, new_len - 1, 1, one, None, kv_len, out, None, ws2)
    torch.cuda.synchronize()
    ref, _ = oracle.tree_attn(inp.q, inp.k, inp.v, "bf16", inp.prefix_len, inp.parent, include_self=True)
    np.testing.assert_allclose(out.float().cpu().numpy().astype(np.float64)[:, 0], ref[:, best], rtol=0, atol=2e-2)
