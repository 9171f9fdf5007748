"""GPU check of dream_accept_path_static, the entry point for callers that cannot allocate: same outputs as
dream_accept_path (bit for bit: all four are integers) and as the oracle, on two calls in a row that share
the library's static scratch, the second on a smaller input; sizes beyond the scratch are rejected on the
host."""
import numpy as np
import pytest

import dream_inputs as di
import oracle

pytestmark = pytest.mark.gpu


def _run_static(dream, torch, gu, logits, dtype, token, parent, max_depth):
    B, T, V = logits.shape
    lg = dream.to_device(logits, dtype)
    tok, par = dream.to_device(token), dream.to_device(parent)
    am = torch.full((B, T), -7, dtype=torch.int32, device="cuda")
    alen = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    path = torch.full((B, max_depth + 1), -7, dtype=torch.int32, device="cuda")
    bonus = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    dream.dream_accept_path_static(lg, gu.DT[dtype], B, T, V, tok, par, max_depth, am, alen, path, bonus)
    torch.cuda.synchronize()
    return am.cpu().numpy(), alen.cpu().numpy(), path.cpu().numpy(), bonus.cpu().numpy()


def test_static_scratch_entry_point_matches_workspace_entry_point_twice():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    import paper_2505_19201_amd as dream
    from tests import gpu_util as gu
    dream.load()
    dream.dream_accept_static_init()
    big = di.Config("static_big", "bf16", 3, 8, 8, 64, 512, 64, 32, 60, 6, 1, 4, 50001, 1, 71)     # 7 chunks per row, ragged tail
    small = di.Config("static_small", "bf16", 1, 8, 8, 64, 512, 64, 32, 24, 4, 1, 4, 9000, 1, 72)   # 2 chunks per row
    for cfg in (big, small):        # the second call reuses the scratch the first one filled
        logits, token, parent, _ = di.accept_inputs(cfg)
        got = _run_static(dream, torch, gu, logits, cfg.dtype, token, parent, cfg.depth)
        ref = gu.run_accept(logits, cfg.dtype, token, parent, cfg.depth)
        want = oracle.accept_path(logits, cfg.dtype, token, parent, cfg.depth)
        for g, r, w in zip(got, ref, want):
            assert np.array_equal(g, r), cfg.name
            assert np.array_equal(g, w), cfg.name


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    import paper_2505_19201_amd as dream
    dream.load()
    one = torch.zeros(16, dtype=torch.int32, device="cuda")
    with pytest.raises(dream.DreamError) as e:     # 64 x 1000 rows of 40 chunks: 2 560 000 partial results
        dream.dream_accept_path_static(one, dream.BF16, 64, 1000, 8192 * 40, one, one, 6, one, one, one, one)
    assert e.value.status == -2 and "static scratch" in str(e.value)
