"""Pins of the oracle's attention entropy (Eq. 2, Section 3.2).  No GPU needed."""
import numpy as np
import pytest

import dream_inputs as di
import oracle


def _cfg(dtype, B=2, Hq=4, Hkv=2, D=64, n=37):
    return di.Config("e", dtype, B, Hq, Hkv, D, Hq * D, n, 0, 1, 0, 1, 2, 100, 1, 30)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_zero_queries_give_uniform_rows_log_count(dtype):
    cfg = _cfg(dtype)
    k = di.verify_inputs(cfg).k
    q = np.zeros_like(di.prefill_q(cfg))
    row, ae = oracle.attention_entropy(q, k, dtype)
    want = np.log(np.arange(1, cfg.prefix + 1))
    np.testing.assert_allclose(row, np.broadcast_to(want, row.shape), atol=1e-12)
    np.testing.assert_allclose(ae, want.mean(), atol=1e-12)
    pos = np.array([[5, 0, 17, 36]] * cfg.batch, dtype=np.int32)
    row, ae = oracle.attention_entropy(q[:, :4], k, dtype, q_pos=pos)
    np.testing.assert_allclose(row, np.broadcast_to(np.log(pos[0] + 1.0), row.shape), atol=1e-12)


def test_a_dominant_key_drives_the_entropy_to_zero_and_bounds_hold():
    cfg = _cfg("f32", B=1, Hq=2, Hkv=2, D=64, n=20)
    q = di.prefill_q(cfg)
    k = di.verify_inputs(cfg).k
    row, _ = oracle.attention_entropy(q, k, "f32")
    assert (row >= -1e-12).all() and (row <= np.log(np.arange(1, 21)) + 1e-12).all()
    assert row[0, :, 0].max() < 1e-12                                    # a single visible key: no uncertainty
    row_sharp, _ = oracle.attention_entropy(q, k, "f32", scale=200.0)    # scores spread far apart: near one-hot rows
    assert row_sharp[0, :, 5:].max() < 1e-3 < row[0, :, 5:].min()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_entropy_is_lse_minus_expected_score_through_the_attention_oracle(dtype):
    """-sum A log A = LSE - sum_j A_j s_j, and sum_j A_j s_j = scale q.(sum_j A_j k_j): the second factor is the
    attention output with V := K.  A chain tree behind an empty prefix makes the attention oracle causal, so
    both terms come from an independently pinned routine."""
    cfg = _cfg(dtype, B=2, Hq=4, Hkv=2, D=64, n=29)
    q = di.prefill_q(cfg)
    k = di.verify_inputs(cfg).k[:, :, :cfg.prefix].copy()
    parents = np.stack([di.chain_tree(cfg.prefix)] * cfg.batch)
    out, lse = oracle.tree_attn(q, k, k, dtype, np.zeros(cfg.batch, dtype=np.int32), parents, include_self=True)
    scale = 1.0 / np.sqrt(cfg.head_dim)
    qf = di.as_f64(q, dtype)
    expected_score = scale * np.einsum("bthd,bthd->bht", qf, out)
    row, ae = oracle.attention_entropy(q, k, dtype)
    np.testing.assert_allclose(row, lse - expected_score, atol=1e-10)
    np.testing.assert_allclose(ae, (lse - expected_score).mean(axis=(1, 2)), atol=1e-10)


def test_against_a_dense_torch_softmax():
    import torch
    cfg = _cfg("f32", B=1, Hq=4, Hkv=2, D=64, n=23)
    q, k = di.prefill_q(cfg), di.verify_inputs(cfg).k
    qt = torch.from_numpy(q.astype(np.float64))[0].permute(1, 0, 2)                       # [Hq, n, D]
    kt = torch.from_numpy(k.astype(np.float64))[0, :, :cfg.prefix].repeat_interleave(2, dim=0)
    s = qt @ kt.transpose(1, 2) / np.sqrt(cfg.head_dim)
    s = s.masked_fill(torch.triu(torch.ones(cfg.prefix, cfg.prefix, dtype=torch.bool), 1), float("-inf"))
    a = torch.softmax(s, dim=-1)
    h = -torch.special.xlogy(a, a).sum(-1)
    row, ae = oracle.attention_entropy(q, k, "f32")
    np.testing.assert_allclose(row[0], h.numpy(), atol=1e-12)
    np.testing.assert_allclose(ae[0], float(h.mean()), atol=1e-12)
