"""GPU parity: dream_project_rows (the linear maps of Eq. 1) against the float64 oracle.

Tolerance: the products of bf16 values are exact in float32 and the MFMA accumulates in float32, so the error is
the bf16 rounding of the stored result: |err| <= 2^-8 |y| + 1e-3.  Cache rows that the call does not address
must keep their bytes."""
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


def _inputs(B, R, hidden, H, D, seed):
    x = di.normal((B, R, hidden), "bf16", seed, di.STREAM_ROWS)
    w32 = di.normal((H * D, hidden), "f32", seed + 1, di.STREAM_ROWS) * np.float32(1.0 / np.sqrt(hidden))
    return x, di.f32_to_bf16_bits(w32)


def _close(got, want):
    err = np.abs(got - want)
    assert (err <= np.abs(want) / 256 + 1e-3).all(), err.max()


@pytest.mark.parametrize("B,R,hidden,H,D", [(1, 1, 4096, 32, 128), (1, 10, 4096, 32, 128), (1, 60, 4096, 32, 128), (2, 7, 5120, 8, 128),
                                            (1, 16, 3840, 16, 256), (8, 10, 2048, 32, 64), (3, 33, 256, 2, 16), (30, 11, 512, 4, 64)])
def test_dense_queries(gu, B, R, hidden, H, D):
    x, w = _inputs(B, R, hidden, H, D, 40 + R)
    got = gu.run_project(x, w, H, D)
    _close(got, oracle.project(x, w, "bf16", H, D))


@pytest.mark.parametrize("B,R,hidden,H,D,with_index", [(1, 7, 4096, 32, 128, False), (2, 10, 4096, 8, 128, True), (4, 20, 2048, 32, 64, True)])
def test_cache_append(gu, B, R, hidden, H, D, with_index):
    x, w = _inputs(B, R, hidden, H, D, 60 + R)
    s_max, T = 150, 40
    cache = di.normal((B, H, s_max, D), "bf16", 77, di.STREAM_K)
    row_base = np.array([90 - 7 * b for b in range(B)], dtype=np.int32)
    g = di.rng(78, 800)
    row_index = np.stack([np.sort(g.choice(T, size=R, replace=False)) for _ in range(B)]).astype(np.int32) if with_index else None
    got = gu.run_project(x, w, H, D, row_base=row_base, row_index=row_index, cache=cache)
    want = oracle.project(x, w, "bf16", H, D)
    touched = np.zeros((B, s_max), dtype=bool)
    for b in range(B):
        for r in range(R):
            row = int(row_base[b]) + (int(row_index[b, r]) if with_index else r)
            touched[b, row] = True
            vals = di.bf16_bits_to_f32(got[b, :, row].view(np.uint16)).astype(np.float64)      # [H, D]
            _close(vals, want[b, r])
    keep = ~touched
    for b in range(B):
        assert np.array_equal(got[b][:, keep[b]], cache[b][:, keep[b]].view(np.int16))         # every other row untouched


def test_identity_weight_copies_rows_exactly(gu):
    hidden = 256
    x = di.normal((2, 5, hidden), "bf16", 91, di.STREAM_ROWS)
    w = di.f32_to_bf16_bits(np.eye(hidden, dtype=np.float32))
    got = gu.run_project(x, w, 4, 64)
    assert np.array_equal(got.reshape(2, 5, hidden), di.as_f64(x, "bf16"))


@pytest.mark.parametrize("B,R,hidden,Hq,Hkv,D", [(1, 10, 5120, 32, 8, 128), (3, 10, 2048, 32, 32, 64), (2, 20, 3840, 16, 8, 256)])
def test_one_launch_for_a_draft_level(gu, B, R, hidden, Hq, Hkv, D):
    e = di.normal((B, R, hidden), "bf16", 101, di.STREAM_ROWS)
    s = di.normal((B, R, hidden), "bf16", 102, di.STREAM_ROWS)
    ws = [di.f32_to_bf16_bits(di.normal((h * D, hidden), "f32", 103 + i, di.STREAM_ROWS) * np.float32(hidden ** -0.5))
          for i, h in enumerate((Hq, Hkv, Hkv))]
    s_max = 120
    kc = di.normal((B, Hkv, s_max, D), "bf16", 110, di.STREAM_K)
    vc = di.normal((B, Hkv, s_max, D), "bf16", 111, di.STREAM_V)
    row_base = np.array([70 - 5 * b for b in range(B)], dtype=np.int32)
    g = di.rng(112, 800)
    row_index = np.stack([np.sort(g.choice(40, size=R, replace=False)) for _ in range(B)]).astype(np.int32)
    q, k, v = gu.run_project_qkv(e, s, ws[0], ws[1], ws[2], Hq, Hkv, D, row_base, row_index, kc, vc)
    _close(q, oracle.project(e, ws[0], "bf16", Hq, D))
    for got, w, cache in ((k, ws[1], kc), (v, ws[2], vc)):
        want = oracle.project(s, w, "bf16", Hkv, D)
        for b in range(B):
            rows = row_base[b] + row_index[b]
            _close(di.bf16_bits_to_f32(got[b][:, rows].view(np.uint16)).astype(np.float64), want[b].transpose(1, 0, 2))
            keep = np.ones(s_max, dtype=bool)
            keep[rows] = False
            assert np.array_equal(got[b][:, keep], cache[b][:, keep].view(np.int16))


def test_rows_outside_the_cache_are_dropped(gu):
    B, R, hidden, H, D, s_max = 1, 6, 256, 2, 64, 20
    x, w = _inputs(B, R, hidden, H, D, 120)
    cache = di.normal((B, H, s_max, D), "bf16", 121, di.STREAM_K)
    row_index = np.array([[0, 1, 2, 3, 4, -40]], dtype=np.int32)          # base 16: rows 16..19, then 20 (out) and -24 (out)
    got = gu.run_project(x, w, H, D, row_base=np.array([16], dtype=np.int32), row_index=row_index, cache=cache)
    want = oracle.project(x, w, "bf16", H, D)
    assert np.array_equal(got[0][:, :16], cache[0][:, :16].view(np.int16))
    for r in range(4):
        _close(di.bf16_bits_to_f32(got[0][:, 16 + r].view(np.uint16)).astype(np.float64), want[0, r])
