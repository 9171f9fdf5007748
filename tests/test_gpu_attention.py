"""GPU parity: dream_tree_verify_attn and dream_draft_xattn against the float64 oracle on identical
seeded inputs.  Tolerances (max-abs): 1e-5 for float32 tensors, 2e-2 for bf16 tensors."""
import numpy as np
import pytest

import dream_inputs as di
import oracle
from tests.attn_cases import (EXTRA_W8_CASES, FULL_VERIFY_PLANS, FULL_XATTN_PLANS, STREAMING_PLANS, VARIANT_CASES, variant_config,
                              variant_prefix_lens)

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from tests import gpu_util
    return gpu_util


def _cfg(name, dtype, B, Hq, Hkv, D, v, q, T, depth, idx):
    return di.Config(name, dtype, B, Hq, Hkv, D, Hq * D, v, q, T, depth, 1, 4, 1000, 1, idx)


def test_tiny_config_verify_all_elements(gu):
    cfg = di.CONFIGS["tiny"]
    x = di.verify_inputs(cfg)
    got, lse = gu.run_verify(x)
    want, want_lse = oracle.tree_attn(x.q, x.k, x.v, cfg.dtype, x.prefix_len, x.parent, True)
    assert np.abs(got - want).max() <= TOL["f32"]
    assert np.abs(lse - want_lse).max() <= 1e-5


SMALL_CASES = [
    # name, B, Hq, Hkv, D, v, q, T, depth, prefix_len, splits
    ("mha128", 2, 4, 4, 128, 150, 43, 60, 6, [193, 101], 0),
    ("mha128_nosplit", 2, 4, 4, 128, 150, 43, 60, 6, [193, 101], 1),
    ("mha128_3split", 1, 2, 2, 128, 300, 77, 60, 6, [377], 3),
    ("gqa4_128", 2, 8, 2, 128, 130, 31, 60, 6, [161, 64], 0),
    ("gqa2_256", 1, 4, 2, 256, 120, 45, 60, 6, [165], 0),
    ("gqa2_256_nosplit", 2, 4, 2, 256, 70, 13, 33, 5, [83, 40], 1),
    ("mha64", 2, 4, 4, 64, 200, 57, 60, 6, [257, 130], 0),
    ("gqa8_64", 1, 8, 1, 64, 100, 30, 64, 6, [130], 2),
    ("t1", 2, 4, 2, 128, 90, 9, 1, 0, [99, 17], 0),
    ("t17", 1, 4, 2, 128, 90, 9, 17, 4, [99], 2),
    ("paper_tree33", 1, 4, 4, 128, 144, 40, 33, 6, [184], 0),
    ("empty_prefix", 1, 2, 2, 64, 0, 0, 20, 4, [0], 0),
    ("long_mha64", 1, 8, 8, 64, 2900, 140, 60, 6, [3040], 0),        # 97 key tiles, still one launch at head_dim 64
    ("long_gqa4_128", 1, 16, 4, 128, 2500, 60, 60, 6, [2560], 0),    # 82 key tiles, grouped queries
    ("longer_mha128", 1, 8, 8, 128, 2500, 60, 60, 6, [2560], 0),     # past the single-launch limit: key splits and merge
    ("pairs320_mha64", 5, 16, 16, 64, 150, 43, 60, 6, [193, 101, 64, 180, 33], 0),   # more (head, tile) pairs than CUs
    ("pairs288_gqa128", 3, 24, 8, 128, 100, 30, 60, 6, [130, 77, 101], 0),            # 12 query tiles per KV head, in pairs
    ("pairs_odd_tiles", 6, 16, 16, 128, 100, 30, 40, 5, [130, 77, 101, 64, 90, 33], 0),   # 3 query tiles per head: a pair with one tile missing
]


@pytest.mark.parametrize("case", SMALL_CASES, ids=[c[0] for c in SMALL_CASES])
def test_bf16_verify_all_elements(gu, case):
    import paper_2505_19201_amd as dream
    name, B, Hq, Hkv, D, v, q, T, depth, pl, splits = case
    cfg = _cfg(name, "bf16", B, Hq, Hkv, D, v, q, T, depth, 40)
    parents = None
    if name == "paper_tree33":
        parents = di.kary_budget_tree()[None]
    x = di.verify_inputs(cfg, prefix_len=pl, parents=parents)
    dream.dream_set_kv_splits(splits)
    try:
        got, lse = gu.run_verify(x)
    finally:
        dream.dream_set_kv_splits(0)
    want, want_lse = oracle.tree_attn(x.q, x.k, x.v, "bf16", x.prefix_len, x.parent, True)
    assert np.isfinite(got).all()
    assert np.abs(got - want).max() <= TOL["bf16"], np.abs(got - want).max()
    assert np.abs(lse - want_lse).max() <= 2e-3


def test_explicit_tree_mask_matches_parent_derived_mask(gu):
    cfg = _cfg("mask", "bf16", 2, 4, 2, 128, 100, 30, 60, 6, 41)
    x = di.verify_inputs(cfg)
    base, _ = gu.run_verify(x)
    masks = np.stack([di.ancestor_mask_bits(x.parent[b], True)[:, 0] for b in range(cfg.batch)])
    got, _ = gu.run_verify(x, tree_mask=masks)
    assert np.array_equal(got, base)
    # a mask that differs from the tree is honoured: pass the star tree's mask with the original parents
    star = di.star_tree(cfg.n_tree)
    star_mask = np.stack([di.ancestor_mask_bits(star, True)[:, 0]] * cfg.batch)
    got2, _ = gu.run_verify(x, tree_mask=star_mask)
    want, _ = oracle.tree_attn(x.q, x.k, x.v, "bf16", x.prefix_len, np.stack([star] * cfg.batch), True)
    assert np.abs(got2 - want).max() <= TOL["bf16"]
    assert np.abs(got2 - base).max() > 1e-3


def test_trees_above_64_nodes(gu):
    """130-node trees (three mask words in use): the mask derived from `parent`, the same mask given explicitly
    ([B, n_tree, 3] words), a foreign explicit mask, and cross-attention levels whose few query rows name nodes of the
    wide tree; float32 tensors as well."""
    cfg = _cfg("wide130", "bf16", 2, 4, 2, 128, 90, 21, 130, 9, 44)
    x = di.verify_inputs(cfg, prefix_len=[111, 60])
    assert gu.verify_plan(x).startswith("attn_bf16_kernel<128,1,1,2,4,4> ")
    base, lse = gu.run_verify(x)
    want, want_lse = oracle.tree_attn(x.q, x.k, x.v, "bf16", x.prefix_len, x.parent, True)
    assert np.abs(base - want).max() <= TOL["bf16"] and np.abs(lse - want_lse).max() <= 2e-3
    masks = np.stack([di.ancestor_mask_bits(x.parent[b], True) for b in range(cfg.batch)])
    assert masks.shape == (cfg.batch, 130, 3)
    got, _ = gu.run_verify(x, tree_mask=masks)
    assert np.array_equal(got, base)
    star = di.star_tree(cfg.n_tree)
    got2, _ = gu.run_verify(x, tree_mask=np.stack([di.ancestor_mask_bits(star, True)] * cfg.batch))
    want2, _ = oracle.tree_attn(x.q, x.k, x.v, "bf16", x.prefix_len, np.stack([star] * cfg.batch), True)
    assert np.abs(got2 - want2).max() <= TOL["bf16"]
    # draft cross-attention: 10 query rows per call that name deep nodes of the wide tree (strict ancestors)
    xx = di.verify_inputs(cfg, prefix_len=[111, 60], streams=(di.STREAM_XQ, di.STREAM_XK, di.STREAM_XV))
    rows = np.stack([np.arange(120, 130, dtype=np.int32)] * cfg.batch)
    gotx, qsel = gu.run_xattn(xx, rows, rows)
    wantx, _ = oracle.tree_attn(qsel, xx.k, xx.v, "bf16", xx.prefix_len, xx.parent, False, q_node=rows)
    assert np.abs(gotx - wantx).max() <= TOL["bf16"]
    # float32 tensors
    cfg32 = _cfg("wide130_f32", "f32", 1, 2, 2, 64, 40, 9, 130, 9, 45)
    x32 = di.verify_inputs(cfg32)
    got32, _ = gu.run_verify(x32)
    want32, _ = oracle.tree_attn(x32.q, x32.k, x32.v, "f32", x32.prefix_len, x32.parent, True)
    assert np.abs(got32 - want32).max() <= TOL["f32"]


def test_seeded_random_shapes_with_the_automatic_plan(gu):
    """48 seeded shapes (batch, head grouping, head_dim, tree size, ragged prefix lengths incl. empty ones) through
    whatever kernel the launch plan picks, every element against the oracle; the set of plans reached is reported."""
    rng = np.random.default_rng(20250519)
    plans = set()
    for i in range(48):
        D = int(rng.choice([64, 128, 256]))
        hkv, g = [(1, 1), (2, 1), (2, 2), (2, 4), (4, 1), (8, 1), (3, 2)][int(rng.integers(7))]
        B = int(rng.integers(1, 6))
        T = int(rng.choice([1, 7, 16, 17, 33, 60, 64, 90]))
        depth = min(6, T - 1)
        prefix = int(rng.choice([0, 5, 31, 32, 100, 257, 700]))
        n_vis = (prefix * 3) // 4
        cfg = di.Config("rand%d" % i, "bf16", B, hkv * g, hkv, D, hkv * g * D, n_vis, prefix - n_vis, T, depth, 1, 4, 1000, 1, 200 + i)
        pl = [prefix] + [int(rng.integers(0, prefix + 1)) for _ in range(B - 1)]
        x = di.verify_inputs(cfg, prefix_len=pl)
        plans.add(gu.verify_plan(x).split(" ")[0])
        got, lse = gu.run_verify(x)
        want, want_lse = oracle.tree_attn(x.q, x.k, x.v, "bf16", x.prefix_len, x.parent, True)
        assert np.isfinite(got).all(), (i, cfg)
        assert np.abs(got - want).max() <= TOL["bf16"], (i, cfg, np.abs(got - want).max())
        assert np.abs(lse - want_lse).max() <= 2e-3, (i, cfg)
    assert len(plans) >= 6, plans


def test_more_query_rows_than_tree_nodes(gu):
    """dream_draft_xattn with 100 query rows that name nodes of a 60-node tree (nodes repeat): every row against the oracle."""
    cfg = _cfg("manyrows", "bf16", 2, 4, 2, 128, 150, 43, 60, 6, 46)
    x = di.verify_inputs(cfg, prefix_len=[193, 80], streams=(di.STREAM_XQ, di.STREAM_XK, di.STREAM_XV))
    rng = np.random.default_rng(5)
    nodes = rng.integers(0, 60, size=(cfg.batch, 100)).astype(np.int32)
    got, qsel = gu.run_xattn(x, nodes, nodes)
    want, _ = oracle.tree_attn(qsel, x.k, x.v, "bf16", x.prefix_len, x.parent, False, q_node=nodes)
    assert np.abs(got - want).max() <= TOL["bf16"]


def test_custom_scale(gu):
    cfg = _cfg("scale", "bf16", 1, 4, 4, 64, 80, 20, 30, 5, 42)
    x = di.verify_inputs(cfg)
    got, _ = gu.run_verify(x, scale=0.05)
    want, _ = oracle.tree_attn(x.q, x.k, x.v, "bf16", x.prefix_len, x.parent, True, scale=0.05)
    assert np.abs(got - want).max() <= TOL["bf16"]


def test_outputs_are_reproducible_bit_for_bit(gu):
    cfg = _cfg("repro", "bf16", 1, 8, 8, 128, 300, 60, 60, 6, 43)
    x = di.verify_inputs(cfg)
    dev = gu.DeviceAttn(x)
    a, la = gu.run_verify(x, dev=dev)
    b, lb = gu.run_verify(x, dev=dev)
    assert np.array_equal(a, b) and np.array_equal(la, lb)


@pytest.mark.parametrize("case", VARIANT_CASES + EXTRA_W8_CASES, ids=[c.variant for c in VARIANT_CASES] + ["extra-" + c.variant for c in EXTRA_W8_CASES])
def test_every_kernel_variant_all_elements(gu, case):
    """One case per bf16 kernel variant the launch plan can choose (tests/test_abi.py checks the list is complete):
    the plan must name that variant, and every output element and log-sum-exp must match the oracle."""
    import paper_2505_19201_amd as dream
    cfg = variant_config(case)
    x = di.verify_inputs(cfg, prefix_len=variant_prefix_lens(case))
    dream.dream_set_kv_splits(case.splits)
    dream.dream_set_q_tiles(case.q_tiles)
    dream.dream_set_tile_waves(case.waves)
    try:
        assert gu.verify_plan(x).startswith(case.variant + " "), gu.verify_plan(x)
        got, lse = gu.run_verify(x)
    finally:
        dream.dream_set_kv_splits(0)
        dream.dream_set_q_tiles(0)
        dream.dream_set_tile_waves(0)
    want, want_lse = oracle.tree_attn(x.q, x.k, x.v, "bf16", x.prefix_len, x.parent, True)
    assert np.isfinite(got).all()
    assert np.abs(got - want).max() <= TOL["bf16"], np.abs(got - want).max()
    assert np.abs(lse - want_lse).max() <= 2e-3


FULL = ["llava", "pixtral", "gemma3", "smolvlm_b1", "smolvlm_b8", "smolvlm_b32"]


@pytest.mark.parametrize("name", FULL)
def test_full_size_verify_all_elements(gu, name):
    """Full measurement shape in the launch configuration bench.py times (asserted by its plan string): every output
    element and every log-sum-exp against the oracle (16 host threads)."""
    cfg = di.CONFIGS[name]
    x = di.verify_inputs(cfg)
    assert gu.verify_plan(x) == FULL_VERIFY_PLANS[name]
    got, lse = gu.run_verify(x)
    oracle.set_threads(16)
    try:
        want, want_lse = oracle.tree_attn(x.q, x.k, x.v, cfg.dtype, x.prefix_len, x.parent, True)
    finally:
        oracle.set_threads(1)
    assert np.isfinite(got).all() and np.isfinite(lse).all()
    assert np.abs(got - want).max() <= TOL["bf16"], np.abs(got - want).max()
    assert np.abs(lse - want_lse).max() <= 2e-3


# ------------------------------------------------------------------------------------------------
# draft cross-attention: strict ancestors, one call per tree level
# ------------------------------------------------------------------------------------------------
def test_tiny_config_xattn_levels(gu):
    cfg = di.CONFIGS["tiny"]
    x = di.xattn_inputs(cfg)
    for lv in di.tree_levels(x.parent[0]):
        rows = lv[None]
        got, qsel = gu.run_xattn(x, rows, rows)
        want, _ = oracle.tree_attn(qsel, x.k, x.v, cfg.dtype, x.prefix_len, x.parent, False, q_node=rows)
        assert np.abs(got - want).max() <= TOL["f32"]


XCASES = [
    ("x_mha128", 2, 4, 4, 128, 150, 43, 60, 6, [193, 101]),
    ("x_gqa4_128", 1, 8, 2, 128, 130, 31, 60, 6, [161]),
    ("x_gqa2_256", 1, 4, 2, 256, 120, 45, 60, 6, [165]),
    ("x_mha64", 2, 4, 4, 64, 200, 57, 60, 6, [257, 130]),
]


@pytest.mark.parametrize("case", XCASES, ids=[c[0] for c in XCASES])
def test_bf16_xattn_levels_all_elements(gu, case):
    name, B, Hq, Hkv, D, v, q, T, depth, pl = case
    cfg = _cfg(name, "bf16", B, Hq, Hkv, D, v, q, T, depth, 44)
    x = di.verify_inputs(cfg, prefix_len=pl, streams=(di.STREAM_XQ, di.STREAM_XK, di.STREAM_XV))
    dev = gu.DeviceAttn(x)
    for lvl in range(depth + 1):
        rows = np.stack([di.tree_levels(x.parent[b])[lvl] for b in range(B)])
        got, qsel = gu.run_xattn(x, rows, rows, dev=dev)
        want, _ = oracle.tree_attn(qsel, x.k, x.v, "bf16", x.prefix_len, x.parent, False, q_node=rows)
        assert np.abs(got - want).max() <= TOL["bf16"]


def test_xattn_all_nodes_in_one_call_without_q_node(gu):
    cfg = _cfg("x_all", "bf16", 1, 4, 4, 128, 100, 28, 60, 6, 45)
    x = di.verify_inputs(cfg)
    rows = np.arange(cfg.n_tree, dtype=np.int32)[None]
    got, qsel = gu.run_xattn(x, rows, None)
    want, _ = oracle.tree_attn(qsel, x.k, x.v, "bf16", x.prefix_len, x.parent, False)
    assert np.abs(got - want).max() <= TOL["bf16"]
    # strict mask differs from the verification mask
    ver, _ = oracle.tree_attn(qsel, x.k, x.v, "bf16", x.prefix_len, x.parent, True)
    assert np.abs(got - ver).max() > 1e-3


def test_xattn_root_with_empty_prefix_gives_zero_row(gu):
    cfg = _cfg("x_empty", "bf16", 1, 2, 2, 64, 0, 0, 12, 3, 46)
    x = di.verify_inputs(cfg, prefix_len=[0])
    rows = np.arange(cfg.n_tree, dtype=np.int32)[None]
    got, qsel = gu.run_xattn(x, rows, rows)
    want, _ = oracle.tree_attn(qsel, x.k, x.v, "bf16", x.prefix_len, x.parent, False, q_node=rows)
    assert np.all(got[0, 0] == 0.0)
    assert np.abs(got - want).max() <= TOL["bf16"]


@pytest.mark.parametrize("name", FULL)
def test_full_size_xattn_round_all_elements(gu, name):
    """One drafting round at the measurement shape: a call per tree level (1,10,10,10,10,10,9 rows), in the launch
    configuration bench.py times (asserted by the plan strings); every output element against the oracle."""
    cfg = di.CONFIGS[name]
    x = di.xattn_inputs(cfg)
    dev = gu.DeviceAttn(x)
    root_plan, level_plan = FULL_XATTN_PLANS[name]
    oracle.set_threads(16)
    try:
        for lvl in range(cfg.depth + 1):
            rows = np.stack([di.tree_levels(x.parent[b])[lvl] for b in range(cfg.batch)])
            if rows.shape[1] in (1, 10):
                assert gu.xattn_plan(x, rows.shape[1]) == (root_plan if rows.shape[1] == 1 else level_plan)
            got, qsel = gu.run_xattn(x, rows, rows, dev=dev)
            want, _ = oracle.tree_attn(qsel, x.k, x.v, cfg.dtype, x.prefix_len, x.parent, False, q_node=rows)
            assert np.isfinite(got).all()
            assert np.abs(got - want).max() <= TOL["bf16"], (lvl, np.abs(got - want).max())
    finally:
        oracle.set_threads(1)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_malformed_device_metadata_stays_in_bounds(gu, dtype):
    """A prefix length past the cache and a parent array with cycles give unspecified numbers but finite ones:
    the kernels clamp the prefix to the cache and treat a parent that does not precede its node as none."""
    cfg = di.Config("bad_meta", dtype, 1, 4, 2, 64, 256, 40, 24, 12, 4, 1, 4, 64, 1, 31)
    x = di.verify_inputs(cfg)
    good, _ = gu.run_verify(x)
    dev = gu.DeviceAttn(x)
    par = x.parent.copy()
    par[0, 3], par[0, 5], par[0, 6], par[0, 7] = 3, 6, 5, 99
    dev.parent = dream_to_device(par)
    dev.prefix_len = dream_to_device(np.array([x.s_max + 1000], dtype=np.int32))
    dev.max_kv = x.s_max
    got, lse = gu.run_verify(x, dev=dev)
    assert np.isfinite(got).all() and np.isfinite(lse).all()
    dev.prefix_len = dream_to_device(np.array([-17], dtype=np.int32))       # clamps to an empty prefix
    got, _ = gu.run_verify(x, dev=dev)
    assert np.isfinite(got).all()
    again, _ = gu.run_verify(x)                                             # and the well-formed call is unaffected
    assert np.array_equal(good, again)


def dream_to_device(a):
    import paper_2505_19201_amd as dream
    return dream.to_device(a)
