"""Pins of the oracle's projections (Eq. 1, Section 3.1: Q = E W_Q, K = S W_K, V = S W_V).  No GPU needed."""
import numpy as np
import pytest

import dream_inputs as di
import oracle


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_identity_and_averaging_weights(dtype):
    B, R, hidden, H, D = 2, 5, 64, 4, 16
    x = di.normal((B, R, hidden), dtype, 1, di.STREAM_ROWS)
    eye = np.eye(hidden, dtype=np.float32)
    w = eye if dtype == "f32" else di.f32_to_bf16_bits(eye)
    y = oracle.project(x, w, dtype, H, D)
    assert np.array_equal(y.reshape(B, R, hidden), di.as_f64(x, dtype))           # W = I: the rows themselves, head-split
    avg = np.full((H * D, hidden), 1.0 / 64, dtype=np.float32)                    # 2^-6 is exact in bf16
    w = avg if dtype == "f32" else di.f32_to_bf16_bits(avg)
    y = oracle.project(x, w, dtype, H, D)
    np.testing.assert_allclose(y, np.broadcast_to(di.as_f64(x, dtype).mean(axis=2)[:, :, None, None], y.shape), atol=1e-14)


def test_row_selectors_transposition_and_linearity():
    B, R, hidden, H, D = 1, 3, 8, 2, 3
    x = di.normal((B, R, hidden), "f32", 2, di.STREAM_ROWS)
    w = np.zeros((H * D, hidden), dtype=np.float32)
    w[0, 5] = 2.0          # output feature 0 (head 0, dim 0) reads twice input feature 5: catches a transposed weight
    w[4, 1] = -1.0         # output feature 4 (head 1, dim 1) reads minus input feature 1
    y = oracle.project(x, w, "f32", H, D)
    want = np.zeros((B, R, H, D))
    want[:, :, 0, 0] = 2.0 * x[:, :, 5]
    want[:, :, 1, 1] = -x[:, :, 1]
    assert np.array_equal(y, want)
    w2 = di.normal((H * D, hidden), "f32", 3, di.STREAM_ROWS)
    x2 = di.normal((B, R, hidden), "f32", 4, di.STREAM_ROWS)
    lhs = oracle.project((x + 2 * x2).astype(np.float32), w2, "f32", H, D)
    rhs = oracle.project(x, w2, "f32", H, D) + 2 * oracle.project(x2, w2, "f32", H, D)
    np.testing.assert_allclose(lhs, rhs, atol=1e-5)


def test_against_a_float64_library_product():
    B, R, hidden, H, D = 2, 7, 96, 3, 32
    x = di.normal((B, R, hidden), "bf16", 5, di.STREAM_ROWS)
    w = di.normal((H * D, hidden), "bf16", 6, di.STREAM_ROWS)
    y = oracle.project(x, w, "bf16", H, D)
    want = np.einsum("brk,nk->brn", di.as_f64(x, "bf16"), di.as_f64(w, "bf16")).reshape(B, R, H, D)
    np.testing.assert_allclose(y, want, atol=1e-12)
