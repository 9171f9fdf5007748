"""GPU parity: dream_spec_accept (acceptance at a sampling temperature) against the float64 oracle.

The integers depend on float comparisons (u against a probability ratio, u against a cumulative sum).  The GPU
works in float32, so a sequence is compared only when the oracle's own run shows every such comparison clear of
float32 error -- decided on the CPU before the GPU result is looked at: |u - min(1, ratio)| > 1e-3 for every
acceptance test and the draw at least 2e-5 of the mass away from both ends of the drawn token's cumulative interval
(the float32 cumulative sums are good to about 1e-6 of the mass).
At least half of the sequences of every case must qualify, and all that qualify must match bit for bit.
A sequence that does not qualify is not waved through: its result must be one of the outcomes the oracle produces when
every too-close comparison on the way is resolved either way (the undecided acceptance tests flipped, the draw landing
on any token of positive probability whose cumulative interval is that close to the drawn point), enumerated on the CPU."""
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


RATIO_EPS, DRAW_EPS = 1e-3, 2e-5


def _clear(detail):
    ok = all(abs(u - min(1.0, r)) > RATIO_EPS for _, r, u in detail["tests"])
    return ok and detail["draw_margin"] > DRAW_EPS


def _legitimate_outcomes(tl64, dl64, token, parent, ua, ub, depth, inv_temperature, limit=64):
    """Every (accept_len, path, bonus) one sequence may legitimately yield: the oracle is re-run with each acceptance
    test that is within RATIO_EPS of its threshold taken either way (a flip changes the walk, so new close calls
    may appear: depth-first over them); the bonus may be any token of positive probability whose cumulative interval
    comes within DRAW_EPS of the drawn point."""
    outcomes, stack, seen = set(), [frozenset()], set()
    while stack and len(seen) < limit:
        flips = stack.pop()
        if flips in seen:
            continue
        seen.add(flips)
        alen, path, bonus, detail = oracle.spec_accept(tl64, dl64, token, parent, ua, ub, depth, inv_temperature=inv_temperature,
                                                       flip_nodes=flips, draw_window=DRAW_EPS)
        for node, ratio, u in detail[0]["tests"]:
            if abs(u - min(1.0, ratio)) <= RATIO_EPS and node not in flips:
                stack.append(flips | {node})
        for t in set(detail[0]["draw_window_tokens"]) | {int(bonus[0])}:
            outcomes.add((int(alen[0]), tuple(path[0].tolist()), t))
    return outcomes


def _draft_children(parent, dl_f64, g):
    """Children tokens drawn without replacement from the draft distribution of their parent (how a sampled draft
    tree is grown); the root's token is arbitrary."""
    B, T, V = dl_f64.shape
    token = np.zeros((B, T), dtype=np.int32)
    for b in range(B):
        for u in range(T):
            kids = np.flatnonzero(parent[b] == u)
            if kids.size:
                x = dl_f64[b, u]
                q = np.exp(x - x.max())
                q /= q.sum()
                token[b, kids] = g.choice(V, size=min(kids.size, V), replace=False, p=q)[:kids.size] if kids.size <= V else 0
    return token


def _case(gu, B, T, depth, V, dtype, seed, spread=2.0, noise=0.7, temperature=1.0, min_clear=0.5, min_compared=0):
    g = di.rng(seed, 700)
    parent = np.stack([di.random_tree(T, depth, seed, b) for b in range(B)]) if T > 1 else np.full((B, 1), -1, dtype=np.int32)
    t32 = di.normal((B, T, V), "f32", seed, di.STREAM_LOGITS) * np.float32(spread)
    d32 = t32 + di.normal((B, T, V), "f32", seed, di.STREAM_DRAFT_LOGITS) * np.float32(noise)
    tl = t32 if dtype == "f32" else di.f32_to_bf16_bits(t32)
    dl = d32 if dtype == "f32" else di.f32_to_bf16_bits(d32)
    tl64, dl64 = di.as_f64(tl, dtype), di.as_f64(dl, dtype)
    token = _draft_children(parent, dl64 / temperature, g)
    ua = g.uniform(size=(B, T)).astype(np.float32)
    ub = g.uniform(size=B).astype(np.float32)
    want_len, want_path, want_bonus, detail = oracle.spec_accept(tl64, dl64, token, parent, ua.astype(np.float64), ub.astype(np.float64),
                                                                depth, inv_temperature=1.0 / temperature)
    clear = np.array([_clear(d) for d in detail])
    assert clear.mean() >= min_clear and clear.sum() >= min_compared, (clear.mean(), clear.sum())
    alen, path, bonus = gu.run_spec_accept(tl, dl, dtype, token, parent, ua, ub, depth, temperature)
    assert (alen >= 0).all() and (alen <= depth).all() and (bonus >= 0).all() and (bonus < V).all()
    assert np.array_equal(alen[clear], want_len[clear]), (alen[clear], want_len[clear])
    assert np.array_equal(path[clear], want_path[clear])
    assert np.array_equal(bonus[clear], want_bonus[clear])
    for b in np.flatnonzero(~clear):      # too close to call in float32: any resolution of the close calls is right, nothing else
        legit = _legitimate_outcomes(tl64[b:b + 1], dl64[b:b + 1], token[b:b + 1], parent[b:b + 1], ua[b:b + 1].astype(np.float64),
                                     ub[b:b + 1].astype(np.float64), depth, 1.0 / temperature)
        assert (int(alen[b]), tuple(path[b].tolist()), int(bonus[b])) in legit, (b, alen[b], path[b], bonus[b], legit)
    _case.last = (parent, detail, clear)
    return alen, clear


def test_worked_example(gu):
    p, q = np.array([0.5, 0.3, 0.2]), np.array([0.2, 0.5, 0.3])
    tl = np.log(p)[None, None].repeat(3, axis=1).astype(np.float32)
    dl = np.log(q)[None, None].repeat(3, axis=1).astype(np.float32)
    parent = np.array([[-1, 0, 0]], dtype=np.int32)
    for tok, ua, ub, want in (([9, 1, 0], [0, 0.5, 0.9], 0.3, (1, [0, 1])), ([9, 1, 0], [0, 0.7, 0.999], 0.3, (1, [0, 2])),
                              ([9, 1, 2], [0, 0.7, 0.0], 0.99, (0, [0, -1]))):
        alen, path, bonus = gu.run_spec_accept(tl, dl, "f32", np.array([tok]), parent, np.array([ua]), np.array([ub]), 6)
        assert alen[0] == want[0] and path[0, :2].tolist() == want[1] and path[0, 2:].tolist() == [-1] * 5
        if want[0] == 0:
            assert bonus[0] == 0
    for u, want in ((0.0, 0), (0.49, 0), (0.51, 1), (0.79, 1), (0.81, 2), (0.999, 2)):
        _, _, bonus = gu.run_spec_accept(tl[:, :1], dl[:, :1], "f32", np.array([[9]]), np.array([[-1]], dtype=np.int32),
                                         np.array([[0.0]]), np.array([u]), 6)
        assert bonus[0] == want


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_cold_limit_is_the_greedy_rule(gu, dtype):
    cfg = di.Config("s", dtype, 8, 4, 4, 64, 256, 8, 8, 40, 5, 1, 2, 5000, 1, 71)
    logits, token, parent, _ = di.accept_inputs(cfg)
    dlog = di.normal(logits.shape, dtype, 72, di.STREAM_DRAFT_LOGITS)
    want_am, want_len, want_path, want_bonus = oracle.accept_path(logits, dtype, token, parent, cfg.depth)
    g = di.rng(73, 701)
    alen, path, bonus = gu.run_spec_accept(logits, dlog, dtype, token, parent, g.uniform(size=token.shape), g.uniform(size=cfg.batch),
                                           cfg.depth, temperature=1.0 / 400.0)
    # a row whose maximum is shared by two tokens (bf16 is coarse) is a fair coin for the sampling rule but not for
    # the greedy one: compare the sequences whose visited rows have a unique maximum
    f = di.as_f64(logits, dtype)
    unique = np.array([all((f[b, n] == f[b, n].max()).sum() == 1 for n in want_path[b] if n >= 0) for b in range(cfg.batch)])
    assert unique.sum() >= cfg.batch // 2
    assert np.array_equal(alen[unique], want_len[unique]) and np.array_equal(path[unique], want_path[unique])
    assert np.array_equal(bonus[unique], want_bonus[unique])


@pytest.mark.parametrize("V", [1, 5, 1000, 1024, 1025, 32003])
def test_ragged_vocabularies(gu, V):
    _case(gu, 16, min(13, max(2, V)), 4, V, "f32", 800 + V)


@pytest.mark.parametrize("dtype,temperature", [("f32", 1.0), ("bf16", 1.0), ("bf16", 0.7)])
def test_trees_of_the_paper_shape(gu, dtype, temperature):
    alen, clear = _case(gu, 48, 33, 6, 4000, dtype, 900, temperature=temperature)
    assert len(set(alen[clear].tolist())) >= 3          # several different accepted depths occur


@pytest.mark.parametrize("name", ["llava", "gemma3"])
def test_full_size_vocabularies(gu, name):
    cfg = di.CONFIGS[name]
    # (at 262144 tokens an interval of the cumulative sum is a few 1e-6 of the mass wide, so few draws are DRAW_EPS clear
    # of both ends: the batch is sized so that at least 8 sequences are compared bit for bit all the same)
    _case(gu, 12 if cfg.vocab <= 65536 else 36, cfg.n_tree, cfg.depth, cfg.vocab, "bf16", cfg.seed, min_clear=0.2, min_compared=8)


def test_largest_tree(gu):
    """1024 nodes per sequence, the most the entry point takes (every per-node table at its full size)."""
    _case(gu, 3, 1024, 12, 777, "f32", 960)


def test_every_branch_of_the_walk_is_exercised(gu):
    """The kernel treats the first rejection at a node symbolically, the second by building arrays, and draws in
    three different ways; the oracle's record of the tests says which of these each compared sequence took."""
    _case(gu, 96, 33, 6, 4000, "bf16", 950, noise=1.0)
    parent, detail, clear = _case.last
    seen = set()
    for b in np.flatnonzero(clear):
        by_node = {}
        for node, ratio, u in detail[b]["tests"]:
            by_node.setdefault(int(parent[b, node]), []).append(u < min(1.0, ratio))
        for outcomes in by_node.values():
            if outcomes[-1]:
                seen.add(("accepted as child number", min(len(outcomes), 3)))
            else:
                seen.add(("all rejected, children", min(len(outcomes), 3)))
        if not by_node or all(o[-1] for o in by_node.values()):
            seen.add(("draw at a node without children",))
    want = {("accepted as child number", 1), ("accepted as child number", 2), ("accepted as child number", 3),
            ("all rejected, children", 1), ("all rejected, children", 2), ("all rejected, children", 3),
            ("draw at a node without children",)}
    assert want <= seen, want - seen
