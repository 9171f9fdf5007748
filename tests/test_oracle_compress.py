"""Pins for the oracle's visual-token scores (Section 3.3 column sums) and top-k selection."""
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

import dream_inputs as di
import oracle

CFG = di.Config("cs", "f32", 2, 4, 2, 16, 64, 9, 6, 4, 2, 1, 2, 50, 1, 21)


def _qk(cfg=CFG, n_q=None, seed=5):
    q = di.prefill_q(cfg, n_q, seed)
    k = di.normal((cfg.batch, cfg.n_kv_heads, cfg.prefix + 3, cfg.head_dim), cfg.dtype, seed, di.STREAM_K)
    return q, k


def _harmonic(m):
    return sum(Fraction(1, i) for i in range(1, m + 1))


@pytest.mark.parametrize("include_diag", [True, False])
def test_zero_query_scores_are_harmonic_differences(include_diag):
    """Q = 0 makes every causal row uniform over its keys, so key j collects 1/(r+1) from every
    row r >= j: score[j] = Hq * (H_P - H_j), or Hq * (H_P - H_{j+1}) without the diagonal."""
    cfg = CFG
    q, k = _qk()
    q[...] = 0
    P = cfg.prefix
    vs, vl = 2, 9
    got = oracle.visual_scores(q, k, "f32", vs, vl, include_diag=include_diag)
    HP = _harmonic(P)
    want = [float(cfg.n_q_heads * (HP - _harmonic(j if include_diag else j + 1))) for j in range(vs, vs + vl)]
    np.testing.assert_allclose(got[0], want, rtol=0, atol=1e-12)
    np.testing.assert_allclose(got[1], want, rtol=0, atol=1e-12)
    assert np.all(np.diff(got[0]) < 0)           # strictly decreasing -> kept set = first k positions
    kept = oracle.topk_keep(got, vs, 1, 3)
    assert kept.tolist() == [[2, 3, 4], [2, 3, 4]]


def test_scores_over_all_keys_sum_to_rows_times_heads():
    cfg = CFG
    q, k = _qk()
    got = oracle.visual_scores(q, k, "f32", 0, cfg.prefix)
    np.testing.assert_allclose(got.sum(axis=1), cfg.n_q_heads * cfg.prefix, atol=1e-11)


def test_scores_equal_dense_causal_softmax_column_sums():
    """Library cross-check: torch softmax over a masked dense score matrix, float64, GQA by
    repeating KV heads; also with explicit (shuffled, partial) row positions."""
    cfg = CFG
    q, k = _qk(seed=9)
    P, G = cfg.prefix, cfg.n_q_heads // cfg.n_kv_heads
    qt = torch.from_numpy(di.as_f64(q, "f32")).permute(0, 2, 1, 3)                      # [B,Hq,P,D]
    kt = torch.from_numpy(di.as_f64(k, "f32"))[:, :, :P].repeat_interleave(G, 1)        # [B,Hq,P,D]
    s = qt @ kt.transpose(-1, -2) / math.sqrt(cfg.head_dim)
    causal = torch.arange(P)[None, :] <= torch.arange(P)[:, None]
    p = torch.softmax(s.masked_fill(~causal, float("-inf")), dim=-1)
    want = p.sum(dim=(1, 2)).numpy()                                                  # [B,P]
    got = oracle.visual_scores(q, k, "f32", 3, 8)
    np.testing.assert_allclose(got, want[:, 3:11], atol=1e-12)
    nodiag = oracle.visual_scores(q, k, "f32", 3, 8, include_diag=False)
    wd = (p * (~torch.eye(P, dtype=torch.bool))).sum(dim=(1, 2)).numpy()
    np.testing.assert_allclose(nodiag, wd[:, 3:11], atol=1e-12)
    # explicit positions: a subset of rows, in shuffled order
    pos = np.stack([di.rng(1, 50, b).permutation(P)[:7] for b in range(cfg.batch)]).astype(np.int32)
    qs = np.stack([q[b, pos[b]] for b in range(cfg.batch)])
    got2 = oracle.visual_scores(qs, k, "f32", 0, P, q_pos=pos)
    for b in range(cfg.batch):
        np.testing.assert_allclose(got2[b], p[b][:, pos[b]].sum(dim=(0, 1)).numpy(), atol=1e-12)


def test_scores_match_value_identity_trick_through_attention_oracle():
    """With V = one-hot rows, attention outputs are the probabilities themselves; a chain tree
    over an empty prefix makes the attention oracle causal, so its summed outputs are the scores."""
    cfg = di.Config("idt", "f32", 1, 2, 2, 8, 16, 6, 0, 6, 5, 1, 2, 10, 1, 22)
    q = di.prefill_q(cfg, 6, 3)
    k = di.normal((1, 2, 6, 8), "f32", 3, di.STREAM_K)
    scores = oracle.visual_scores(q, k, "f32", 0, 6)
    v = np.zeros((1, 2, 6, 8), dtype=np.float32)
    for j in range(6):
        v[0, :, j, j] = 1.0
    out, _ = oracle.tree_attn(q, k, v, "f32", [0], di.chain_tree(6)[None], True)
    np.testing.assert_allclose(scores[0], out[0].sum(axis=(0, 1))[:6], atol=1e-12)


def test_keep_count_rounds_to_nearest_half_up():
    assert oracle.keep_count(5, 1, 2) == 3 and oracle.keep_count(7, 1, 4) == 2 and oracle.keep_count(6, 1, 4) == 2
    assert oracle.keep_count(576, 1, 4) == 144 and oracle.keep_count(1088, 1, 4) == 272
    assert oracle.keep_count(576, 3, 4) == 432                # the paper's own 75 % operating point
    for v in range(0, 40):
        for den in range(1, 9):
            for num in range(0, den + 1):
                want = math.floor(Fraction(v * num, den) + Fraction(1, 2))
                assert oracle.keep_count(v, num, den) == min(max(want, 0), v)
                assert (v * num + den // 2) // den == want    # the integer form the library documents


def test_topk_equals_the_unique_dominating_subset():
    """Exhaustive: of all k-subsets exactly one has every member beating every non-member under
    (higher score, then lower index); the oracle must return it, ascending, offset by vis_start."""
    g = di.rng(4, di.STREAM_SCORES)
    for trial in range(30):
        v = int(g.integers(1, 9))
        s = g.integers(0, 4, size=v).astype(np.float64) * 0.5          # many exact ties
        for num, den in ((1, 2), (1, 4), (3, 4), (0, 1), (1, 1)):
            k = oracle.keep_count(v, num, den)
            good = []
            for sub in itertools.combinations(range(v), k):
                inside = set(sub)
                ok = all((s[i] > s[j]) or (s[i] == s[j] and i < j)
                         for i in inside for j in range(v) if j not in inside)
                if ok:
                    good.append(list(sub))
            assert len(good) == 1
            got = oracle.topk_keep(s[None], 10, num, den)
            assert got.shape == (1, k) and got[0].tolist() == [10 + i for i in good[0]]


def test_topk_edge_cases():
    s = np.full((2, 12), 0.25)
    assert oracle.topk_keep(s, 5, 1, 3).tolist() == [[5, 6, 7, 8]] * 2          # all equal -> first k
    assert oracle.topk_keep(s, 5, 0, 3).shape == (2, 0)
    assert oracle.topk_keep(s, 5, 3, 3).tolist() == [list(range(5, 17))] * 2
    s2 = np.array([[0.1, 0.9, 0.5, 0.9, 0.2, 0.5]])
    assert oracle.topk_keep(s2, 0, 1, 2).tolist() == [[1, 2, 3]]                # tie 0.5: index 2 beats 5


def test_gather_rows_is_a_row_copy():
    cfg = di.Config("g", "bf16", 2, 2, 2, 8, 24, 6, 2, 4, 2, 1, 2, 10, 1, 23)
    src = di.feature_rows(cfg)
    kept = np.array([[0, 3, 7], [1, 2, 6]], dtype=np.int32)
    got = oracle.gather_rows(src, "bf16", kept)
    for b in range(2):
        assert np.array_equal(got[b], src[b, kept[b]])


@pytest.mark.parametrize("name", ["llava", "pixtral", "gemma3", "smolvlm_b1"])
def test_diagonal_reading_report(name, record_property, capsys):
    """Section 3.3 sums a token's attention weights "across all other tokens"; the library includes the diagonal term
    A_jj (a reading of this build).  This reports, on the seeded full-size inputs, how many kept indices change when
    the diagonal is excluded, and checks what must hold either way: the two scores differ by the diagonal terms, one in
    [0, 1] per head."""
    cfg = di.CONFIGS[name]
    q, k = di.prefill_q(cfg), di.verify_inputs(cfg).k
    oracle.set_threads(8)
    try:
        with_diag = oracle.visual_scores(q, k, cfg.dtype, 0, cfg.n_visual)
        without = oracle.visual_scores(q, k, cfg.dtype, 0, cfg.n_visual, include_diag=False)
    finally:
        oracle.set_threads(1)
    gap = with_diag - without
    assert (gap >= -1e-12).all() and (gap <= cfg.n_q_heads + 1e-12).all()
    kept_a = oracle.topk_keep(with_diag, 0, cfg.keep_num, cfg.keep_den)
    kept_b = oracle.topk_keep(without, 0, cfg.keep_num, cfg.keep_den)
    assert kept_a.shape == kept_b.shape
    changed = int(sum(len(set(kept_a[b]) - set(kept_b[b])) for b in range(cfg.batch)))
    record_property("kept", int(kept_a.shape[1]))
    record_property("kept_indices_that_change_without_the_diagonal", changed)
    with capsys.disabled():
        print(f"\n[diagonal reading] {name}: {kept_a.shape[1]} of {cfg.n_visual} visual tokens kept; "
              f"{changed} kept indices change when A_jj is excluded")
