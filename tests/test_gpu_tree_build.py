"""GPU parity: dream_tree_expand_level and dream_tree_finalize against the oracle.

Tokens are decided by comparing the logits themselves, so they are bit-exact.  Scores are float32 on the GPU
(log-sum-exp over up to 262144 terms with fast exp/log) against float64: |error| <= 1e-4 at |score| <~ 30.
Where a float32 score decides an integer (the next frontier, the final rerank) the check is two-layered, as for
the visual top-k: (i) the GPU's ranking equals the oracle's ranking of the GPU's own float32 scores bit for bit;
(ii) end to end the integers equal the oracle's whenever the oracle's scores around the cut are further apart
than the float32 error (asserted before the GPU result is looked at)."""
import numpy as np
import pytest

import dream_inputs as di
import oracle

pytestmark = pytest.mark.gpu
SCORE_TOL = 1e-4
GAP = 1e-3


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from tests import gpu_util
    return gpu_util


def _rank(values):
    return np.lexsort((np.arange(values.shape[0]), -values))


def _check_level(gu, logits, dtype, cum, k, need_gap=True):
    tok, sc, nxt = gu.run_expand(logits, dtype, cum, k)
    want_tok, want_sc, want_nxt = oracle.expand_level(di.as_f64(logits, dtype), cum.astype(np.float64), k)
    assert np.array_equal(tok, want_tok)
    assert np.abs(sc - want_sc).max() <= SCORE_TOL, np.abs(sc - want_sc).max()
    B, F, _ = tok.shape
    kf = nxt.shape[1]
    for b in range(B):
        assert np.array_equal(nxt[b], _rank(sc[b].reshape(-1).astype(np.float64))[:kf])       # (i)
        s = np.sort(want_sc[b].reshape(-1))[::-1]
        if kf < s.shape[0] and s[kf - 1] - s[kf] > GAP:
            assert sorted(nxt[b].tolist()) == sorted(want_nxt[b].tolist())                     # (ii) same set
    return tok, sc, nxt


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("vocab", [1, 5, 1000, 8191, 8192, 8193, 32003])
def test_ragged_vocabularies(gu, dtype, vocab):
    k = min(4, vocab)
    logits, cum = di.draft_level_inputs(2, 3, vocab, dtype, 900 + vocab, level=2)
    _check_level(gu, logits, dtype, cum, k)


@pytest.mark.parametrize("name,F,k", [("llava", 10, 10), ("llava", 4, 4), ("pixtral", 10, 10), ("gemma3", 16, 16), ("smolvlm_b8", 10, 10)])
def test_config_vocabularies_and_widths(gu, name, F, k):
    cfg = di.CONFIGS[name]
    for level in (0, 3):
        f = 1 if level == 0 else F
        logits, cum = di.draft_level_inputs(cfg.batch, f, cfg.vocab, cfg.dtype, cfg.seed, level=level)
        _check_level(gu, logits, cfg.dtype, cum, k)


def test_exact_ties_resolve_toward_lower_indices(gu):
    V, F, k = 20000, 4, 6
    logits = np.zeros((1, F, V), dtype=np.float32)                 # all equal: tokens 0..k-1, all scores cum - log V
    cum = np.array([[-1.0, -1.0, -2.0, -1.0]], dtype=np.float32)
    tok, sc, nxt = gu.run_expand(logits, "f32", cum, k)
    assert tok[0].tolist() == [list(range(k))] * F
    np.testing.assert_allclose(sc[0], np.broadcast_to(cum[0][:, None] - np.log(V), (F, k)), atol=SCORE_TOL)
    assert nxt[0].tolist() == [0, 1, 2, 3, 4, 5]                   # rows 0, 1, 3 tie: lowest flat indices first
    logits[0, :, 17000] = 3.0
    logits[0, :, 9000] = 3.0                                       # two equal maxima in different chunks
    tok, sc, nxt = gu.run_expand(logits, "f32", cum, k)
    assert tok[0, 0].tolist() == [9000, 17000, 0, 1, 2, 3]


@pytest.mark.parametrize("levels", [40, 200, 3000])
def test_heavily_tied_logits(gu, levels):
    """Logits drawn from a small set of values: the candidate lists of the selection hold from a handful to
    hundreds of equal values (both of its paths), and ties must still resolve toward lower token indices."""
    V, F, k = 20000, 3, 10
    g = di.rng(500 + levels, 401)
    logits = (g.integers(0, levels, size=(2, F, V)) * (8.0 / levels)).astype(np.float32)
    cum = np.zeros((2, F), dtype=np.float32)
    tok, sc, _ = gu.run_expand(logits, "f32", cum, k)
    want_tok, want_sc, _ = oracle.expand_level(logits.astype(np.float64), cum.astype(np.float64), k)
    assert np.array_equal(tok, want_tok)
    assert np.abs(sc - want_sc).max() <= SCORE_TOL


def test_finalize_bit_exact_including_ties(gu):
    g = di.rng(77, 400)
    for N, budget in [(85, 32), (85, 100), (2, 1), (1, 5), (1024, 59), (601, 600), (333, 0)]:
        B = 3
        parent = np.zeros((B, N), dtype=np.int32)
        score = np.zeros((B, N), dtype=np.float32)
        for b in range(B):
            parent[b, 0] = -1
            for i in range(1, N):
                parent[b, i] = int(g.integers(0, i))
                # scores shrink along a path; coarse steps make many exact ties
                score[b, i] = score[b, parent[b, i]] - np.float32(int(g.integers(0, 4)) * 0.25)
        token = g.integers(0, 50000, size=(B, N)).astype(np.int32)
        n_tree, par, tok, pidx = gu.run_finalize(score, parent, token, budget)
        T, want_par, want_tok, want_pidx = oracle.finalize_tree(score.astype(np.float64), parent, token, budget)
        assert n_tree == T
        assert np.array_equal(pidx, want_pidx) and np.array_equal(par, want_par) and np.array_equal(tok, want_tok)


@pytest.mark.parametrize("V,dtype,k,depth,budget,seed", [(40, "f32", 4, 6, 32, 1), (300, "bf16", 4, 6, 32, 2), (32000, "bf16", 10, 6, 59, 3)])
def test_whole_tree_level_by_level_matches_the_oracle(gu, V, dtype, k, depth, budget, seed):
    """Drives the GPU entry points the way a decoder would: a synthetic draft (next-token logits drawn per
    (level, parent token) from a seeded table) is evaluated for the frontier, one expansion call per level, the
    pool grows on the host, one finalize call at the end.  The oracle runs the same draft in float64."""
    # the first seed of a fixed list whose oracle run has every cut clear of float32 error (decided on the CPU,
    # before the GPU result exists)
    for attempt in range(5):
        base = di.normal((depth, 64, V), dtype, 5000 + seed + 100 * attempt, di.STREAM_DRAFT_LOGITS)

        def draft_bits(path, base=base):                           # logits stored in `dtype`, picked by level and last token
            return base[len(path) - 1, path[-1] % 64]

        want = oracle.build_tree(lambda p: di.as_f64(draft_bits(p), dtype), root_token=3, k=k, depth=depth, budget=budget)
        s = np.sort(want["pool_score"][1:])[::-1]
        keep_n = min(budget, s.shape[0])
        if (keep_n == s.shape[0] or s[keep_n - 1] - s[keep_n] > GAP) and want["frontier_gap"] > GAP:
            break
    else:
        pytest.fail("no seed with clear cuts")
    pool_score, pool_parent, pool_token = [0.0], [-1], [3]
    frontier = [0]
    for level in range(depth):
        paths = []
        for f in frontier:
            p, a = [], f
            while a >= 0:
                p.append(pool_token[a])
                a = pool_parent[a]
            paths.append(p[::-1])
        logits = np.stack([draft_bits(p) for p in paths])[None]
        cum = np.asarray([[pool_score[f] for f in frontier]], dtype=np.float32)
        tok, sc, nxt = gu.run_expand(logits, dtype, cum, k)
        start = len(pool_score)
        for fi, f in enumerate(frontier):
            for j in range(k):
                pool_score.append(float(sc[0, fi, j]))
                pool_parent.append(f)
                pool_token.append(int(tok[0, fi, j]))
        frontier = [start + int(i) for i in nxt[0]]
    ps = np.asarray(pool_score, dtype=np.float32)[None]
    n_tree, par, tok, pidx = gu.run_finalize(ps, np.asarray(pool_parent, dtype=np.int32)[None],
                                             np.asarray(pool_token, dtype=np.int32)[None], budget)
    assert n_tree == want["n_tree"]
    assert par[0, 0] == -1 and all(0 <= par[0, i] < i for i in range(1, n_tree))
    assert len(pool_score) == want["pool_score"].shape[0]
    if True:
        got_paths, want_paths = set(), set()
        for tree_par, tree_tok, dst in ((par[0], tok[0], got_paths), (want["parent"], want["token"], want_paths)):
            for i in range(1, n_tree):
                seq, a = [], i
                while a > 0:
                    seq.append(int(tree_tok[a]))
                    a = int(tree_par[a])
                dst.add(tuple(seq[::-1]))
        # every cut of the oracle's run is clear of float32 error (asserted above), so the kept token paths agree
        assert got_paths == want_paths
        np.testing.assert_allclose(np.sort(ps[0, pidx[0, 1:]])[::-1], np.sort(want["pool_score"][want["pool_index"][1:]])[::-1],
                                   atol=10 * SCORE_TOL)
