"""Host-side checks of the seeded input generators (no method arithmetic involved)."""
import os

import numpy as np

import dream_inputs as di


def _golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")
    out = {}
    for line in open(path):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = int(line[1])
    return out


def test_bf16_rounding_is_nearest_even():
    # 1 + 2^-8 is exactly halfway between bf16 neighbours 1.0 and 1 + 2^-7: ties go to even (1.0)
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -2.5, 0.0], dtype=np.float32)
    back = di.bf16_bits_to_f32(di.f32_to_bf16_bits(x))
    assert back.tolist() == [1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -2.5, 0.0]
    # agrees with torch's conversion on random data
    import torch
    r = di.rng(1, 99).standard_normal(10000, dtype=np.float32)
    t = torch.from_numpy(r).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(t, di.f32_to_bf16_bits(r))


def test_config_trees_shape():
    for name, cfg in di.CONFIGS.items():
        for seq in range(min(cfg.batch, 3)):
            p = di.config_tree(cfg, seq)
            assert p.shape == (cfg.n_tree,) and p[0] == -1
            assert all(0 <= p[i] < i for i in range(1, cfg.n_tree))
            assert di.tree_depths(p).max() == cfg.depth
    a, b = di.config_tree(di.CONFIGS["smolvlm_b8"], 0), di.config_tree(di.CONFIGS["smolvlm_b8"], 1)
    assert not np.array_equal(a, b)          # every sequence has its own tree
    p = di.config_tree(di.CONFIGS["llava"])
    assert (p == 0).sum() == 10              # root top-10 branching


def test_paper_shaped_tree_matches_stated_setup():
    g = _golden()
    p = di.kary_budget_tree(g["tree_children_k"], g["tree_depth"], g["max_draft_tokens"])
    assert len(p) - 1 == g["max_draft_tokens"]
    assert di.tree_depths(p).max() == g["tree_depth"]
    assert np.bincount(p[1:]).max() <= g["tree_children_k"]
    assert di.tree_depths(p).max() + 1 == g["max_tokens_per_round"]


def test_sibling_tokens_distinct_and_mask_bits():
    p = di.config_tree(di.CONFIGS["llava"])
    tok = di.tree_tokens(p, 32000, 7)
    for a in range(len(p)):
        kids = tok[p == a]
        assert len(set(kids.tolist())) == len(kids)
    m = di.ancestor_mask_bits(p, True)
    ms = di.ancestor_mask_bits(p, False)
    for i in range(len(p)):
        assert (int(m[i, 0]) >> i) & 1 == 1 and (int(ms[i, 0]) >> i) & 1 == 0
        assert int(m[i, 0]) == int(ms[i, 0]) | (1 << i)
        assert bin(int(m[i, 0])).count("1") == di.tree_depths(p)[i] + 1


def test_generators_are_deterministic():
    a = di.verify_inputs(di.CONFIGS["tiny"])
    b = di.verify_inputs(di.CONFIGS["tiny"])
    assert np.array_equal(a.q, b.q) and np.array_equal(a.k, b.k) and np.array_equal(a.parent, b.parent)
    assert a.s_max == 96 + 8 + 5 and np.all(a.k[:, :, 104:, :] == np.float32(3.0e4))
