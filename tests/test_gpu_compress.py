"""GPU parity: dream_visual_compress.  Stage B (top-k keep) is bit-exact on identical float32 scores;
stage A scores are compared to the float64 oracle; end-to-end kept indices are bit-exact on seeds whose
k-th / (k+1)-th oracle scores are separated by more than the float32 evaluation error (the seed is
screened on the oracle side only, before the GPU result is looked at)."""
import numpy as np
import pytest

import dream_inputs as di
import oracle

pytestmark = pytest.mark.gpu

GAP = 1e-4      # minimum relative gap between the k-th and (k+1)-th oracle score for an end-to-end index check
SCORE_RTOL = {"f32": 2e-5, "bf16": 2e-4}


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from tests import gpu_util
    return gpu_util


def _qk(cfg, seed, n_q=None, extra_rows=3):
    q = di.prefill_q(cfg, n_q, seed)
    k = di.normal((cfg.batch, cfg.n_kv_heads, cfg.prefix + extra_rows, cfg.head_dim), cfg.dtype, seed, di.STREAM_K)
    return q, k


def _boundary_gap(scores64, k):
    """Smallest relative gap over the batch between the last kept and the first dropped score."""
    worst = np.inf
    for row in scores64:
        s = np.sort(row)[::-1]
        if 0 < k < len(s):
            worst = min(worst, (s[k - 1] - s[k]) / abs(s[k - 1]))
    return worst


def _pick_seed(cfg, vis_start, vis_len, q_pos=None):
    """First seed of a fixed list whose oracle scores have a safe gap at the keep boundary."""
    k = oracle.keep_count(vis_len, cfg.keep_num, cfg.keep_den)
    for seed in [cfg.seed + 1000 * i for i in range(5)]:
        q, kk = _qk(cfg, seed)
        want = oracle.visual_scores(q, kk, cfg.dtype, vis_start, vis_len, q_pos=q_pos)
        if _boundary_gap(want, k) > GAP:
            return seed, q, kk, want
    raise AssertionError("no seed with a safe top-k boundary")


def test_stage_b_is_bit_exact_on_given_scores(gu):
    g = di.rng(11, di.STREAM_SCORES)
    cases = [(1, 1, 1, 2), (3, 5, 1, 2), (2, 64, 1, 4), (2, 576, 1, 4), (4, 1088, 1, 4), (1, 1025, 3, 4), (2, 2500, 1, 3),
             (1, 16384, 1, 4), (2, 37, 0, 1), (2, 37, 1, 1)]
    for (B, v, num, den) in cases:
        s = g.standard_normal(size=(B, v), dtype=np.float32)
        s[:, ::3] = np.float32(0.5)                               # a third of the entries tie exactly
        s[0, : v // 2] = np.round(s[0, : v // 2] * 2) / 2          # coarse values: many more ties
        _, kept, _ = gu.run_compress("bf16", None, None, 0, 7, v, num, den, scores_in=s)
        want = oracle.topk_keep(s, 7, num, den)
        assert np.array_equal(kept, want), (B, v, num, den)


def test_tiny_config_scores_kept_and_gather(gu):
    cfg = di.CONFIGS["tiny"]
    seed, q, k, want = _pick_seed(cfg, 0, cfg.n_visual)
    rows = di.feature_rows(cfg, seed=seed)
    scores, kept, gathered = gu.run_compress(cfg.dtype, q, k, cfg.prefix, 0, cfg.n_visual, cfg.keep_num, cfg.keep_den,
                                             gather_src=rows)
    np.testing.assert_allclose(scores, want, rtol=SCORE_RTOL["f32"])
    want_kept = oracle.topk_keep(want, 0, cfg.keep_num, cfg.keep_den)
    assert kept.shape == (1, 32) and np.array_equal(kept, want_kept)
    assert np.array_equal(gathered, oracle.gather_rows(rows, cfg.dtype, want_kept))
    # stage B alone on the GPU's own float32 scores
    assert np.array_equal(kept, oracle.topk_keep(scores, 0, cfg.keep_num, cfg.keep_den))


SMALL = [
    # name, B, Hq, Hkv, D, v, q_text, vis_start, keep
    ("mha128", 2, 4, 4, 128, 150, 43, 0, (1, 4)),
    ("gqa4_128_offset", 1, 8, 2, 128, 130, 61, 20, (1, 2)),
    ("gqa2_256", 1, 4, 2, 256, 100, 37, 5, (3, 4)),
    ("mha64", 2, 4, 4, 64, 200, 57, 9, (1, 4)),
]


@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
def test_bf16_scores_and_kept_small(gu, case):
    name, B, Hq, Hkv, D, v, qt, vs, (num, den) = case
    cfg = di.Config(name, "bf16", B, Hq, Hkv, D, 64, v, qt, 8, 3, num, den, 100, 1, 60)
    seed, q, k, want = _pick_seed(cfg, vs, v)
    rows = di.feature_rows(cfg, seed=seed)
    scores, kept, gathered = gu.run_compress("bf16", q, k, cfg.prefix, vs, v, num, den, gather_src=rows)
    np.testing.assert_allclose(scores, want, rtol=SCORE_RTOL["bf16"])
    want_kept = oracle.topk_keep(want, vs, num, den)
    assert np.array_equal(kept, want_kept)
    assert np.array_equal(kept, oracle.topk_keep(scores, vs, num, den))
    assert np.array_equal(gathered, oracle.gather_rows(rows, "bf16", want_kept))


def test_explicit_row_positions(gu):
    cfg = di.Config("pos", "bf16", 2, 4, 2, 128, 64, 90, 30, 8, 3, 1, 2, 100, 1, 61)
    P = cfg.prefix
    n_q = 50
    pos = np.stack([np.sort(di.rng(5, 903, b).permutation(P)[:n_q])[::-1] for b in range(cfg.batch)]).astype(np.int32)
    q = di.prefill_q(cfg, n_q, 8)
    k = di.normal((cfg.batch, cfg.n_kv_heads, P + 2, cfg.head_dim), "bf16", 8, di.STREAM_K)
    want = oracle.visual_scores(q, k, "bf16", 10, 80, q_pos=pos)
    scores, kept, _ = gu.run_compress("bf16", q, k, P, 10, 80, 1, 2, q_pos=pos)
    np.testing.assert_allclose(scores, want, rtol=SCORE_RTOL["bf16"], atol=1e-6)
    assert np.array_equal(kept, oracle.topk_keep(scores, 10, 1, 2))


def test_scores_are_reproducible_bit_for_bit(gu):
    cfg = di.Config("rep", "bf16", 1, 8, 8, 128, 64, 300, 84, 8, 3, 1, 4, 100, 1, 62)
    q, k = _qk(cfg, 3)
    a, ka, _ = gu.run_compress("bf16", q, k, cfg.prefix, 0, 300, 1, 4)
    b, kb, _ = gu.run_compress("bf16", q, k, cfg.prefix, 0, 300, 1, 4)
    assert np.array_equal(a, b) and np.array_equal(ka, kb)


def test_zero_keep_and_zero_span(gu):
    cfg = di.Config("z", "bf16", 1, 4, 4, 64, 64, 40, 10, 8, 3, 0, 1, 100, 1, 63)
    q, k = _qk(cfg, 4)
    scores, kept, _ = gu.run_compress("bf16", q, k, cfg.prefix, 0, 40, 0, 1)
    assert kept.shape == (1, 0) and np.isfinite(scores).all()
    scores, kept, _ = gu.run_compress("bf16", q, k, cfg.prefix, 0, 0, 1, 2, want_scores=False)
    assert kept.shape == (1, 0)


@pytest.mark.parametrize("name", ["llava", "pixtral", "gemma3", "smolvlm_b1", "smolvlm_b8"])
def test_full_size_configs(gu, name):
    """Measurement shapes, all prefill rows: scores against the oracle, kept indices and gathered rows
    bit-exact (seed screened for a safe boundary gap on the oracle side)."""
    cfg = di.CONFIGS[name]
    oracle.set_threads(min(16, oracle.hw_threads()))
    try:
        seed, q, k, want = _pick_seed(cfg, 0, cfg.n_visual)
    finally:
        oracle.set_threads(1)
    rows = di.feature_rows(cfg, seed=seed)
    scores, kept, gathered = gu.run_compress("bf16", q, k, cfg.prefix, 0, cfg.n_visual, cfg.keep_num, cfg.keep_den,
                                             gather_src=rows)
    np.testing.assert_allclose(scores, want, rtol=SCORE_RTOL["bf16"])
    want_kept = oracle.topk_keep(want, 0, cfg.keep_num, cfg.keep_den)
    assert kept.shape[1] == oracle.keep_count(cfg.n_visual, cfg.keep_num, cfg.keep_den)
    assert np.array_equal(kept, want_kept)
    assert np.array_equal(kept, oracle.topk_keep(scores, 0, cfg.keep_num, cfg.keep_den))
    assert np.array_equal(gathered, oracle.gather_rows(rows, "bf16", want_kept))


def test_full_size_smolvlm_b32(gu):
    """32 sequences per call, all prefill rows.  Scores of every sequence against the oracle; the kept set is the exact
    top-k of the library's own float32 scores for every sequence, and equals the oracle's kept set wherever the
    oracle's boundary gap is safe (decided per sequence on the oracle side; most sequences must qualify)."""
    cfg = di.CONFIGS["smolvlm_b32"]
    q, k = _qk(cfg, cfg.seed)
    oracle.set_threads(min(16, oracle.hw_threads()))
    try:
        want = oracle.visual_scores(q, k, cfg.dtype, 0, cfg.n_visual)
    finally:
        oracle.set_threads(1)
    n_keep = oracle.keep_count(cfg.n_visual, cfg.keep_num, cfg.keep_den)
    safe = np.array([_boundary_gap(want[b:b + 1], n_keep) > GAP for b in range(cfg.batch)])
    assert safe.sum() >= cfg.batch // 2
    rows = di.feature_rows(cfg)
    scores, kept, gathered = gu.run_compress("bf16", q, k, cfg.prefix, 0, cfg.n_visual, cfg.keep_num, cfg.keep_den, gather_src=rows)
    np.testing.assert_allclose(scores, want, rtol=SCORE_RTOL["bf16"])
    assert np.array_equal(kept, oracle.topk_keep(scores, 0, cfg.keep_num, cfg.keep_den))
    want_kept = oracle.topk_keep(want, 0, cfg.keep_num, cfg.keep_den)
    assert np.array_equal(kept[safe], want_kept[safe])
    assert np.array_equal(gathered, oracle.gather_rows(rows, "bf16", kept))


def _causal_row_lse(q, k, dtype, scale=None, q_pos=None):
    """Natural-log sum of exp of the scaled scores of every row over keys 0..pos(row), float64 numpy: [B, Hq, n_q].
    (What an attention kernel with a log-sum-exp output leaves; written out here so that nothing comes from the GPU.)"""
    qf, kf = di.as_f64(q, dtype), di.as_f64(k, dtype)
    B, n_q, Hq, D = qf.shape
    Hkv = kf.shape[1]
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    out = np.empty((B, Hq, n_q))
    for b in range(B):
        pos = np.arange(n_q) if q_pos is None else np.asarray(q_pos)[b]
        for h in range(Hq):
            s = qf[b, :, h, :] @ kf[b, h // (Hq // Hkv)].T * scale            # [n_q, n_keys]
            s = np.where(np.arange(s.shape[1])[None, :] <= pos[:, None], s, -np.inf)
            m = s.max(axis=1)
            out[b, h] = m + np.log(np.exp(s - m[:, None]).sum(axis=1))
    return out


@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
def test_caller_supplied_row_lse_small(gu, case):
    """With the rows' log-sum-exps given, stage A is one pass: same scores (to tolerance) and the same kept set."""
    name, B, Hq, Hkv, D, v, qt, vs, (num, den) = case
    cfg = di.Config(name, "bf16", B, Hq, Hkv, D, 64, v, qt, 8, 3, num, den, 100, 1, 60)
    seed, q, k, want = _pick_seed(cfg, vs, v)
    lse = _causal_row_lse(q, k, "bf16")
    scores, kept, _ = gu.run_compress("bf16", q, k, cfg.prefix, vs, v, num, den, row_lse=lse)
    np.testing.assert_allclose(scores, want, rtol=SCORE_RTOL["bf16"])
    assert np.array_equal(kept, oracle.topk_keep(want, vs, num, den))


def test_caller_supplied_row_lse_tiny_f32_and_positions(gu):
    cfg = di.CONFIGS["tiny"]
    seed, q, k, want = _pick_seed(cfg, 0, cfg.n_visual)
    lse = _causal_row_lse(q, k, "f32")
    scores, kept, _ = gu.run_compress("f32", q, k, cfg.prefix, 0, cfg.n_visual, cfg.keep_num, cfg.keep_den, row_lse=lse)
    np.testing.assert_allclose(scores, want, rtol=SCORE_RTOL["f32"])
    assert np.array_equal(kept, oracle.topk_keep(want, 0, cfg.keep_num, cfg.keep_den))
    # explicit, shuffled row positions (bf16)
    c2 = di.Config("pos_lse", "bf16", 2, 4, 2, 128, 512, 100, 60, 8, 3, 1, 2, 100, 1, 62)
    q, k = _qk(c2, 5, n_q=90)
    g = di.rng(63, 902)
    q_pos = np.stack([g.permutation(c2.prefix)[:90] for _ in range(c2.batch)]).astype(np.int32)
    want = oracle.visual_scores(q, k, "bf16", 10, 80, q_pos=q_pos)
    lse = _causal_row_lse(q, k, "bf16", q_pos=q_pos)
    scores, kept, _ = gu.run_compress("bf16", q, k, c2.prefix, 10, 80, 1, 2, q_pos=q_pos, row_lse=lse)
    np.testing.assert_allclose(scores, want, rtol=SCORE_RTOL["bf16"])


@pytest.mark.parametrize("name", ["llava", "gemma3"])
def test_caller_supplied_row_lse_full_size(gu, name):
    cfg = di.CONFIGS[name]
    oracle.set_threads(min(16, oracle.hw_threads()))
    try:
        seed, q, k, want = _pick_seed(cfg, 0, cfg.n_visual)
    finally:
        oracle.set_threads(1)
    lse = _causal_row_lse(q, k, "bf16")
    scores, kept, _ = gu.run_compress("bf16", q, k, cfg.prefix, 0, cfg.n_visual, cfg.keep_num, cfg.keep_den, row_lse=lse)
    np.testing.assert_allclose(scores, want, rtol=SCORE_RTOL["bf16"])
    assert np.array_equal(kept, oracle.topk_keep(want, 0, cfg.keep_num, cfg.keep_den))
