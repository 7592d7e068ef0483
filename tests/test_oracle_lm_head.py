"""Pins for oracle_lm_head: it is a matrix product, so the library matmul and exact special cases pin it."""
import numpy as np
import torch


def _bits(x):
    return torch.as_tensor(x, dtype=torch.float32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def _f64(bits):
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64)


def test_matches_library_matmul(oracle):
    rng = np.random.default_rng(0)
    hidden, W = _bits(rng.normal(0, 0.02, (7, 96))), _bits(rng.normal(0, 0.02, (53, 96)))
    got = oracle.lm_head(hidden, W)
    ref = (_f64(hidden) @ _f64(W).T).numpy()
    assert got.shape == (7, 53)
    np.testing.assert_allclose(got, ref, rtol=1e-6, atol=1e-9)


def test_identity_weight_returns_hidden_exactly(oracle):
    rng = np.random.default_rng(1)
    hidden = _bits(rng.normal(0, 1, (5, 32)))
    W = _bits(np.eye(32))
    assert np.array_equal(oracle.lm_head(hidden, W), _f64(hidden).float().numpy())


def test_one_hot_hidden_selects_weight_columns(oracle):
    """hidden = e_k picks column k of W: catches a transposed operand or wrong stride (V != H)."""
    rng = np.random.default_rng(2)
    W = _bits(rng.normal(0, 1, (11, 6)))
    hidden = _bits(np.eye(6)[[4, 0]])
    got = oracle.lm_head(hidden, W)
    Wf = _f64(W).float().numpy()
    assert np.array_equal(got[0], Wf[:, 4]) and np.array_equal(got[1], Wf[:, 0])
