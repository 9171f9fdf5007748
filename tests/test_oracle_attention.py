"""Pins for the oracle's masked attention (verification, include_self) and cross-attention
(strict ancestors).  Every expectation here is built without the oracle: a library SDPA in
float64, closed forms, or a dense-mask implementation that derives the mask by transitive
closure instead of walking parents."""
import numpy as np
import pytest
import torch

import dream_inputs as di
import oracle

SMALL = di.Config("small", "f32", 2, 4, 2, 16, 64, 10, 7, 9, 4, 1, 2, 50, 1, 11)


def _inputs(cfg=SMALL, parents=None, prefix_len=None, seed=123):
    return di.verify_inputs(cfg, seed=seed, parents=parents, prefix_len=prefix_len)


def _closure_mask(parent, include_self):
    """[T,T] bool: m[i,a] iff a is an ancestor of i (or i itself): boolean closure of the
    child->parent relation by repeated squaring."""
    T = len(parent)
    A = np.zeros((T, T), dtype=bool)
    for i in range(1, T):
        A[i, parent[i]] = True
    R = A.copy()
    for _ in range(T):
        R = R | (R.astype(int) @ A.astype(int) > 0)
    return R | np.eye(T, dtype=bool) if include_self else R


def _dense_reference(x, cfg, include_self, q_node=None, scale=None):
    """Dense masked softmax attention in float64 numpy over the full S = s_max key range."""
    B, Tq, Hq, D = x.q.shape
    G = Hq // x.k.shape[1]
    q, k, v = (di.as_f64(a, cfg.dtype) for a in (x.q, x.k, x.v))
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    out = np.zeros((B, Tq, Hq, D))
    lse = np.zeros((B, Hq, Tq))
    for b in range(B):
        P = int(x.prefix_len[b])
        tm = _closure_mask(x.parent[b], include_self)
        mask = np.zeros((Tq, x.s_max), dtype=bool)
        for i in range(Tq):
            node = i if q_node is None else int(q_node[b][i])
            mask[i, :P] = True
            mask[i, P:P + len(x.parent[b])] = tm[node]
        for h in range(Hq):
            s = scale * q[b, :, h, :] @ k[b, h // G].T
            s = np.where(mask, s, -np.inf)
            m = s.max(axis=1, keepdims=True)
            e = np.exp(s - m)
            z = e.sum(axis=1, keepdims=True)
            out[b, :, h, :] = (e / z) @ np.where(np.isfinite(v[b, h // G]), v[b, h // G], 0.0)
            lse[b, h] = (m + np.log(z))[:, 0]
    return out, lse


def test_chain_tree_is_dense_causal_attention_sdpa():
    """A chain is a legal tree: rows must equal causal attention of T new tokens over P+T keys.
    Expectation from torch's scaled_dot_product_attention in float64 (GQA via head repetition)."""
    cfg = SMALL
    parents = np.stack([di.chain_tree(cfg.n_tree)] * cfg.batch)
    x = _inputs(parents=parents, prefix_len=[17, 11])
    got, _ = oracle.tree_attn(x.q, x.k, x.v, cfg.dtype, x.prefix_len, x.parent, True)
    G = cfg.n_q_heads // cfg.n_kv_heads
    for b in range(cfg.batch):
        P, T = int(x.prefix_len[b]), cfg.n_tree
        q = torch.from_numpy(di.as_f64(x.q[b], cfg.dtype)).permute(1, 0, 2)[None]          # [1,Hq,T,D]
        k = torch.from_numpy(di.as_f64(x.k[b, :, :P + T], cfg.dtype)).repeat_interleave(G, 0)[None]
        v = torch.from_numpy(di.as_f64(x.v[b, :, :P + T], cfg.dtype)).repeat_interleave(G, 0)[None]
        causal = torch.arange(P + T)[None, :] <= (P + torch.arange(T))[:, None]
        want = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=causal)[0].permute(1, 0, 2)
        np.testing.assert_allclose(got[b], want.numpy(), rtol=0, atol=1e-12)


def test_single_node_tree_is_plain_decode_attention():
    cfg = di.Config("one", "f32", 1, 2, 2, 8, 16, 5, 3, 1, 0, 1, 2, 10, 1, 12)
    x = _inputs(cfg, parents=np.array([[-1]], dtype=np.int32))
    got, lse = oracle.tree_attn(x.q, x.k, x.v, cfg.dtype, x.prefix_len, x.parent, True)
    q, k, v = (di.as_f64(a, "f32") for a in (x.q, x.k, x.v))
    for h in range(2):
        s = (k[0, h, :9] @ q[0, 0, h]) / np.sqrt(8)
        w = np.exp(s - s.max())
        np.testing.assert_allclose(got[0, 0, h], (w / w.sum()) @ v[0, h, :9], atol=1e-13)
        np.testing.assert_allclose(lse[0, h, 0], np.log(np.exp(s).sum()), atol=1e-12)


def test_star_tree_rows_see_prefix_root_and_self_only():
    cfg = SMALL
    parents = np.stack([di.star_tree(cfg.n_tree)] * cfg.batch)
    x = _inputs(parents=parents)
    got, _ = oracle.tree_attn(x.q, x.k, x.v, cfg.dtype, x.prefix_len, x.parent, True)
    q, k, v = (di.as_f64(a, "f32") for a in (x.q, x.k, x.v))
    P = cfg.prefix
    for i in (1, 4, 8):
        rows = list(range(P)) + [P] + [P + i]
        for h in range(cfg.n_q_heads):
            s = k[1, h // 2, rows] @ q[1, i, h] / np.sqrt(cfg.head_dim)
            w = np.exp(s - s.max())
            np.testing.assert_allclose(got[1, i, h], (w / w.sum()) @ v[1, h // 2, rows], atol=1e-13)


@pytest.mark.parametrize("include_self", [True, False])
def test_random_tree_against_dense_closure_mask(include_self):
    cfg = SMALL
    parents = np.stack([di.random_tree(cfg.n_tree, 4, 5, b) for b in range(cfg.batch)])
    x = _inputs(parents=parents, prefix_len=[12, 17])
    got, lse = oracle.tree_attn(x.q, x.k, x.v, cfg.dtype, x.prefix_len, x.parent, include_self)
    want, want_lse = _dense_reference(x, cfg, include_self)
    np.testing.assert_allclose(got, want, atol=1e-12)
    np.testing.assert_allclose(lse, want_lse, atol=1e-12)


def test_bf16_inputs_are_widened_exactly_and_scale_is_used():
    cfg = di.Config("smallb", "bf16", 1, 4, 2, 16, 64, 10, 7, 9, 4, 1, 2, 50, 1, 13)
    x = _inputs(cfg)
    got, _ = oracle.tree_attn(x.q, x.k, x.v, "bf16", x.prefix_len, x.parent, True, scale=0.37)
    want, _ = _dense_reference(x, cfg, True, scale=0.37)
    np.testing.assert_allclose(got, want, atol=1e-12)
    other, _ = oracle.tree_attn(x.q, x.k, x.v, "bf16", x.prefix_len, x.parent, True)
    assert np.abs(other - got).max() > 1e-3          # default scale 1/sqrt(D) = 0.25 differs from 0.37


@pytest.mark.parametrize("include_self", [True, False])
def test_zero_query_gives_mean_of_visible_value_rows(include_self):
    cfg = SMALL
    x = _inputs()
    x.q[...] = 0
    got, lse = oracle.tree_attn(x.q, x.k, x.v, cfg.dtype, x.prefix_len, x.parent, include_self)
    v = di.as_f64(x.v, "f32")
    for b in range(cfg.batch):
        P = int(x.prefix_len[b])
        for i in range(cfg.n_tree):
            anc = di.path_to(x.parent[b], i)
            if not include_self:
                anc = anc[:-1]
            rows = list(range(P)) + [P + a for a in anc]
            for h in range(cfg.n_q_heads):
                np.testing.assert_allclose(got[b, i, h], v[b, h // 2, rows].mean(axis=0), atol=1e-13)
                np.testing.assert_allclose(lse[b, h, i], np.log(len(rows)), atol=1e-13)


def test_constant_value_rows_give_that_constant():
    x = _inputs()
    x.v[...] = np.float32(-1.75)
    got, _ = oracle.tree_attn(x.q, x.k, x.v, "f32", x.prefix_len, x.parent, True)
    np.testing.assert_allclose(got, -1.75, atol=1e-13)


def test_prefix_permutation_and_sibling_relabelling_invariance():
    cfg = SMALL
    x = _inputs()
    base, _ = oracle.tree_attn(x.q, x.k, x.v, "f32", x.prefix_len, x.parent, True)
    perm = di.rng(3, 77).permutation(cfg.prefix)
    k2, v2 = x.k.copy(), x.v.copy()
    k2[:, :, :cfg.prefix] = x.k[:, :, perm]
    v2[:, :, :cfg.prefix] = x.v[:, :, perm]
    again, _ = oracle.tree_attn(x.q, k2, v2, "f32", x.prefix_len, x.parent, True)
    np.testing.assert_allclose(again, base, atol=1e-13)
    # swap two leaves' labels (nodes T-1 and T-2): q rows, K/V rows and parent entries move together
    T, P = cfg.n_tree, cfg.prefix
    a, c = T - 1, T - 2
    par = x.parent.copy()
    assert not (par == a).any() and not (par == c).any()
    par[:, [a, c]] = par[:, [c, a]]
    q3, k3, v3 = x.q.copy(), x.k.copy(), x.v.copy()
    q3[:, [a, c]] = x.q[:, [c, a]]
    k3[:, :, [P + a, P + c]] = x.k[:, :, [P + c, P + a]]
    v3[:, :, [P + a, P + c]] = x.v[:, :, [P + c, P + a]]
    # parent[a] < a must still hold for the relabelled tree
    if all(par[b, a] < a and par[b, c] < c for b in range(cfg.batch)):
        sw, _ = oracle.tree_attn(q3, k3, v3, "f32", x.prefix_len, par, True)
        np.testing.assert_allclose(sw[:, a], base[:, c], atol=1e-13)
        np.testing.assert_allclose(sw[:, c], base[:, a], atol=1e-13)
        np.testing.assert_allclose(sw[:, :c], base[:, :c], atol=1e-13)


def test_lse_normalises_the_visible_scores():
    cfg = SMALL
    x = _inputs()
    _, lse = oracle.tree_attn(x.q, x.k, x.v, "f32", x.prefix_len, x.parent, True)
    q, k = di.as_f64(x.q, "f32"), di.as_f64(x.k, "f32")
    b, h, i = 1, 3, 6
    P = int(x.prefix_len[b])
    rows = list(range(P)) + [P + a for a in di.path_to(x.parent[b], i)]
    s = k[b, h // 2, rows] @ q[b, i, h] / np.sqrt(cfg.head_dim)
    assert abs(np.exp(s - lse[b, h, i]).sum() - 1.0) < 1e-12


def test_xattn_root_query_sees_only_target_rows_and_levels_use_q_node():
    cfg = SMALL
    x = _inputs(seed=321)
    levels = di.tree_levels(x.parent[0])
    # same tree in both sequences for this test
    x.parent[1] = x.parent[0]
    q, k, v = (di.as_f64(a, "f32") for a in (x.q, x.k, x.v))
    P = cfg.prefix
    for lv in levels:
        qn = np.stack([lv, lv])
        ql = np.ascontiguousarray(x.q[:, lv])
        got, _ = oracle.tree_attn(ql, x.k, x.v, "f32", x.prefix_len, x.parent, False, q_node=qn)
        for r, node in enumerate(lv):
            rows = list(range(P)) + [P + a for a in di.path_to(x.parent[0], node)[:-1]]
            if node == 0:
                assert rows == list(range(P))
            s = k[0, 1, rows] @ q[0, node, 2] / np.sqrt(cfg.head_dim)
            w = np.exp(s - s.max())
            np.testing.assert_allclose(got[0, r, 2], (w / w.sum()) @ v[0, 1, rows], atol=1e-13)


@pytest.mark.parametrize("include_self", [True, False])
def test_invisible_rows_cannot_leak(include_self):
    """Blow up K and V of every tree row a query must not see; its output must not move."""
    cfg = SMALL
    x = _inputs(seed=55)
    base, _ = oracle.tree_attn(x.q, x.k, x.v, "f32", x.prefix_len, x.parent, include_self)
    P = cfg.prefix
    for i in (0, 3, cfg.n_tree - 1):
        vis = set(di.path_to(x.parent[0], i))
        if not include_self:
            vis.discard(i)
        k2, v2 = x.k.copy(), x.v.copy()
        for a in range(cfg.n_tree):
            if a not in vis:
                k2[0, :, P + a] = 1.0e3
                v2[0, :, P + a] = -7.0e3
        got, _ = oracle.tree_attn(x.q, k2, v2, "f32", x.prefix_len, x.parent, include_self)
        np.testing.assert_allclose(got[0, i], base[0, i], atol=1e-13)
    # and a visible row does matter
    k2 = x.k.copy()
    k2[0, :, P + 0] += 1.0
    moved, _ = oracle.tree_attn(x.q, k2, x.v, "f32", x.prefix_len, x.parent, True)
    assert np.abs(moved[0] - base[0]).max() > 1e-6 if include_self else True


def test_empty_visible_set_gives_zero_row():
    cfg = di.Config("empty", "f32", 1, 2, 2, 8, 16, 0, 0, 3, 2, 1, 2, 10, 1, 14)
    x = di.verify_inputs(cfg, prefix_len=[0], parents=np.array([[-1, 0, 1]], dtype=np.int32))
    got, lse = oracle.tree_attn(x.q, x.k, x.v, "f32", x.prefix_len, x.parent, False)
    assert np.all(got[0, 0] == 0.0) and np.all(np.isneginf(lse[0, :, 0]))
    assert np.all(np.isfinite(lse[0, :, 1:]))


def test_attn_row_matches_batched_entry():
    x = _inputs()
    full, lse = oracle.tree_attn(x.q, x.k, x.v, "f32", x.prefix_len, x.parent, True)
    row, l1 = oracle.attn_row(x.q, x.k, x.v, "f32", x.prefix_len, x.parent, True, b=1, h=2, row=5)
    assert np.array_equal(row, full[1, 5, 2]) and l1 == lse[1, 2, 5]
