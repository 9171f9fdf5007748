"""Pins of the oracle's stochastic tree acceptance (Section 2.1 rule at temperature > 0).  No GPU needed.

The defining property of the rule -- the emitted token follows the TARGET distribution whatever the draft -- is
checked by Monte Carlo with children drawn from the draft by this test (not by the oracle); the cold limit must
reproduce the greedy acceptance oracle for any random numbers; one case is worked out by hand."""
import numpy as np
import pytest

import dream_inputs as di
import oracle


def test_worked_example():
    # V = 3, root with two children.  target p = (.5,.3,.2), draft q = (.2,.5,.3)
    p, q = np.array([0.5, 0.3, 0.2]), np.array([0.2, 0.5, 0.3])
    tl = np.log(p)[None, None].repeat(3, axis=1)
    dl = np.log(q)[None, None].repeat(3, axis=1)
    parent = np.array([[-1, 0, 0]], dtype=np.int32)
    # child 1 proposes token 1: ratio .3/.5 = .6
    alen, path, bonus, _ = oracle.spec_accept(tl, dl, np.array([[9, 1, 0]]), parent, np.array([[0, 0.5, 0.9]]), np.array([0.3]), 6)
    assert alen[0] == 1 and path[0, :2].tolist() == [0, 1]
    # u = .7 rejects it: target becomes max(p-q,0) = (.3,0,0) -> (1,0,0); draft without token 1 -> (.4,0,.6);
    # child 2 proposes token 0: ratio 1/.4 > 1 -> accepted whatever u
    alen, path, bonus, d = oracle.spec_accept(tl, dl, np.array([[9, 1, 0]]), parent, np.array([[0, 0.7, 0.999]]), np.array([0.3]), 6)
    assert alen[0] == 1 and path[0, :2].tolist() == [0, 2]
    assert [round(t[1], 12) for t in d[0]["tests"]] == [0.6, 2.5]
    # if child 2 proposes token 2 instead: residual target has no mass there -> rejected -> bonus from (1,0,0): token 0
    alen, path, bonus, _ = oracle.spec_accept(tl, dl, np.array([[9, 1, 2]]), parent, np.array([[0, 0.7, 0.0]]), np.array([0.99]), 6)
    assert alen[0] == 0 and path[0].tolist() == [0, -1, -1, -1, -1, -1, -1] and bonus[0] == 0
    # no children at all: the bonus is the inverse CDF of p: u < .5 -> 0, .5 <= u < .8 -> 1, else 2
    for u, want in ((0.0, 0), (0.49, 0), (0.51, 1), (0.79, 1), (0.81, 2), (0.999, 2)):
        _, _, bonus, _ = oracle.spec_accept(tl[:, :1], dl[:, :1], np.array([[9]]), np.array([[-1]], dtype=np.int32), np.array([[0.0]]),
                                            np.array([u]), 6)
        assert bonus[0] == want


def test_forced_resolutions_of_close_calls_on_the_worked_example():
    """flip_nodes and draw_window (used by the GPU test to enumerate what float32 may legitimately decide when a
    comparison is too close to call) do what they say on the hand-worked case, and nothing when not asked."""
    p, q = np.array([0.5, 0.3, 0.2]), np.array([0.2, 0.5, 0.3])
    tl = np.log(p)[None, None].repeat(3, axis=1)
    dl = np.log(q)[None, None].repeat(3, axis=1)
    parent = np.array([[-1, 0, 0]], dtype=np.int32)
    tok, ua, ub = np.array([[9, 1, 0]]), np.array([[0, 0.5, 0.9]]), np.array([0.3])
    base = oracle.spec_accept(tl, dl, tok, parent, ua, ub, 6)
    same = oracle.spec_accept(tl, dl, tok, parent, ua, ub, 6, flip_nodes=frozenset(), draw_window=0.0)
    assert all(np.array_equal(a, b) for a, b in zip(base[:3], same[:3]))
    # u = .5 < .6 accepts child 1; flipped, it is rejected and child 2 (ratio 2.5) is accepted instead
    alen, path, _, d = oracle.spec_accept(tl, dl, tok, parent, ua, ub, 6, flip_nodes=frozenset({1}))
    assert alen[0] == 1 and path[0, :2].tolist() == [0, 2] and [round(t[1], 12) for t in d[0]["tests"]] == [0.6, 2.5]
    # flipping both leaves no accepted child: the draw comes from the residual (1,0,0)
    alen, path, bonus, _ = oracle.spec_accept(tl, dl, tok, parent, ua, ub, 6, flip_nodes=frozenset({1, 2}))
    assert alen[0] == 0 and bonus[0] == 0
    # a lone root: u = .51 draws token 1 of (.5,.3,.2), 0.01 above the end of token 0's interval and 0.29 below token 2's
    one = (tl[:, :1], dl[:, :1], np.array([[9]]), np.array([[-1]], dtype=np.int32), np.array([[0.0]]), np.array([0.51]), 6)
    for window, want in ((0.0, [1]), (0.005, [1]), (0.02, [0, 1]), (0.3, [0, 1, 2])):
        _, _, bonus, d = oracle.spec_accept(*one, draw_window=window)
        assert bonus[0] == 1 and d[0]["draw_window_tokens"] == want
    # tokens of zero probability are never candidates: p = (.5, 0, .5), u = .5 sits on the boundary
    tz = np.log(np.array([0.5, 1e-300, 0.5]))[None, None]
    tz[0, 0, 1] = -np.inf
    _, _, bonus, d = oracle.spec_accept(tz, tz, one[2], one[3], one[4], np.array([0.5]), 6, draw_window=0.01)
    assert bonus[0] == 2 and d[0]["draw_window_tokens"] == [0, 2]


@pytest.mark.parametrize("m", [1, 2, 3])
def test_the_emitted_token_follows_the_target_distribution(m):
    """One level, m children drawn without replacement from the draft distribution: whatever the draft, the first
    token of the round (the accepted child's, else the bonus) must be distributed like the target."""
    V, N = 6, 60000
    g = di.rng(11 + m, 600)
    p = g.dirichlet(np.ones(V) * 0.7)
    q = g.dirichlet(np.ones(V) * 0.7)
    T = 1 + m
    tl = np.broadcast_to(np.log(p), (N, T, V)).copy()
    dl = np.broadcast_to(np.log(q), (N, T, V)).copy()
    parent = np.broadcast_to(np.array([-1] + [0] * m, dtype=np.int32), (N, T)).copy()
    token = np.zeros((N, T), dtype=np.int64)
    for n in range(N):
        token[n, 1:] = g.choice(V, size=m, replace=False, p=q)
    ua, ub = g.uniform(size=(N, T)), g.uniform(size=N)
    alen, path, bonus, _ = oracle.spec_accept(tl, dl, token, parent, ua, ub, max_depth=1)
    first = np.where(alen > 0, token[np.arange(N), np.maximum(path[:, 1], 0)], bonus)
    freq = np.bincount(first, minlength=V) / N
    assert np.abs(freq - p).max() < 4 * np.sqrt(0.25 / N) + 1e-3, (freq, p)
    assert 0.05 < (alen > 0).mean() < 1.0


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_cold_limit_is_the_greedy_acceptance(dtype):
    cfg = di.Config("s", dtype, 4, 4, 4, 64, 256, 8, 8, 24, 5, 1, 2, 400, 1, 60)
    logits, token, parent, ends = di.accept_inputs(cfg)
    tl = di.as_f64(logits, dtype)
    dl = di.as_f64(di.normal(logits.shape, dtype, 61, di.STREAM_DRAFT_LOGITS), dtype)
    want_am, want_len, want_path, want_bonus = oracle.accept_path(logits, dtype, token, parent, cfg.depth)
    for trial in range(3):
        g = di.rng(62, 601, trial)
        ua, ub = g.uniform(size=token.shape), g.uniform(size=cfg.batch)
        alen, path, bonus, _ = oracle.spec_accept(tl, dl, token, parent, ua, ub, cfg.depth, inv_temperature=400.0)
        assert np.array_equal(alen, want_len) and np.array_equal(path, want_path) and np.array_equal(bonus, want_bonus)


def test_identical_models_accept_every_first_child():
    cfg = di.Config("s", "f32", 2, 4, 4, 64, 256, 8, 8, 30, 4, 1, 2, 300, 1, 63)
    logits, token, parent, _ = di.accept_inputs(cfg)
    tl = di.as_f64(logits, "f32")
    g = di.rng(64, 602)
    alen, path, bonus, _ = oracle.spec_accept(tl, tl, token, parent, g.uniform(size=token.shape), g.uniform(size=2), cfg.depth)
    for b in range(2):
        cur, d = 0, 0
        while d < cfg.depth:
            kids = np.flatnonzero(parent[b] == cur)
            if kids.size == 0:
                break
            cur, d = int(kids[0]), d + 1
            assert path[b, d] == cur
        assert alen[b] == d
