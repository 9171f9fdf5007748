"""GPU parity: dream_attention_entropy (Eq. 2) against the float64 oracle.

Tolerance: the entropy is LSE minus the attention-weighted mean score, two float32 sums over up to ~1600 keys of
exact bf16 products, values of order 1..10: |error| <= 2e-4 (bf16 tensors), 2e-5 (float32 tensors)."""
import numpy as np
import pytest

import dream_inputs as di
import oracle

pytestmark = pytest.mark.gpu
TOL = {"f32": 2e-5, "bf16": 2e-4}


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from tests import gpu_util
    return gpu_util


def _check(gu, cfg, n_q=None, q_pos=None, scale=None):
    q = di.prefill_q(cfg, n_q=n_q)
    k = di.verify_inputs(cfg).k
    n_keys = cfg.prefix
    row, ae = gu.run_entropy(cfg.dtype, q, k, n_keys, q_pos=q_pos, scale=0.0 if scale is None else scale)
    want_row, want_ae = oracle.attention_entropy(q, k, cfg.dtype, q_pos=q_pos, scale=scale)
    assert np.isfinite(row).all()
    assert np.abs(row - want_row).max() <= TOL[cfg.dtype], np.abs(row - want_row).max()
    assert np.abs(ae - want_ae).max() <= TOL[cfg.dtype]
    return row, ae


def test_tiny_f32(gu):
    _check(gu, di.CONFIGS["tiny"])


@pytest.mark.parametrize("Hq,Hkv,D,n", [(4, 4, 64, 200), (8, 2, 128, 333), (4, 2, 256, 97), (2, 1, 64, 1), (4, 4, 128, 65)])
def test_small_bf16_shapes_span_tiles_and_ragged_tails(gu, Hq, Hkv, D, n):
    cfg = di.Config("e", "bf16", 2, Hq, Hkv, D, Hq * D, n, 0, 4, 2, 1, 2, 100, 1, 31)
    _check(gu, cfg)


def test_explicit_positions_and_scale(gu):
    cfg = di.Config("e", "bf16", 2, 4, 2, 128, 512, 150, 0, 4, 2, 1, 2, 100, 1, 32)
    pos = np.stack([di.rng(5, 500, b).integers(0, 150, size=40) for b in range(2)]).astype(np.int32)
    _check(gu, cfg, n_q=40, q_pos=pos, scale=0.31)
    cfg32 = di.Config("e", "f32", 1, 4, 4, 64, 256, 90, 0, 4, 2, 1, 2, 100, 1, 33)
    _check(gu, cfg32, n_q=17, q_pos=np.arange(17, dtype=np.int32)[None] * 5)


def test_zero_queries_reproduce_log_count(gu):
    cfg = di.Config("e", "bf16", 1, 4, 4, 128, 512, 300, 0, 4, 2, 1, 2, 100, 1, 34)
    q = np.zeros_like(di.prefill_q(cfg))
    k = di.verify_inputs(cfg).k
    row, ae = gu.run_entropy("bf16", q, k, 300)
    np.testing.assert_allclose(row, np.broadcast_to(np.log(np.arange(1, 301)), row.shape), atol=TOL["bf16"])


@pytest.mark.parametrize("name", ["llava", "pixtral", "gemma3", "smolvlm_b8"])
def test_full_size_configs(gu, name):
    cfg = di.CONFIGS[name]
    _check(gu, cfg)
