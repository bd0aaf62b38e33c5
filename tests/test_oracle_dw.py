"""Pins for the oracle's weight gradient (Eq. 2, Alg. 1 lines 11-12) and Gradient Importance (Eq. 4) -- CPU only."""
import numpy as np
import pytest
import torch

import oracle


def _bf16(x):
    return torch.from_numpy(np.asarray(x, dtype=np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def _bf16_to_f64(b):
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _f64(a):
    return a.astype(np.float64) if a.dtype == np.float32 else _bf16_to_f64(a)


def _dense_pruned(a, g, r):
    vals, mask, _, _ = oracle.prune_pack(a, g, r)
    keep = np.unpackbits(mask.view(np.uint8), bitorder="little")[:a.size].astype(bool)
    return vals, mask, np.where(keep, _f64(a.reshape(-1)), 0.0)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_linear_ratio0_is_dense_matmul_and_ratio1_is_zero(dtype):
    rng = np.random.default_rng(0)
    M, K, N = 37, 48, 29  # non-square: a transposed operand or output fails
    A = rng.standard_normal((M, K)).astype(np.float32)
    dY = rng.standard_normal((M, N)).astype(np.float32)
    if dtype == "bf16":
        A, dY = _bf16(A), _bf16(dY)
    vals, mask, _, _ = oracle.prune_pack(A, K, 0.0)
    dW = oracle.dw_linear(vals, mask, dY, M, K, N)
    ref = _f64(dY).T @ _f64(A)  # library float64 matmul: dW = dY^T A, [N, K]
    assert dW.shape == (N, K)
    assert np.array_equal(dW, ref.astype(np.float32)) or np.allclose(dW, ref, rtol=1e-6, atol=1e-6)
    vals, mask, _, _ = oracle.prune_pack(A, K, 1.0)
    assert not oracle.dw_linear(vals, mask, dY, M, K, N).any()


@pytest.mark.parametrize("r", [0.3, 0.5, 0.9])
def test_linear_pruned_matches_masked_matmul_and_linearity(r):
    rng = np.random.default_rng(1)
    M, K, N = 50, 64, 24
    A = rng.standard_normal((M, K)).astype(np.float32)
    dY = rng.standard_normal((M, N)).astype(np.float32)
    vals, mask, Ad = _dense_pruned(A, K, r)
    dW = oracle.dw_linear(vals, mask, dY, M, K, N)
    ref = dY.astype(np.float64).T @ Ad.reshape(M, K)
    assert np.allclose(dW, ref, rtol=1e-6, atol=1e-6)
    # linearity: dW(pruned) = dW(dense) - dW(dropped part)
    dense = dY.astype(np.float64).T @ A.astype(np.float64)
    dropped = dY.astype(np.float64).T @ (A.astype(np.float64) - Ad.reshape(M, K))
    assert np.allclose(dW, dense - dropped, rtol=1e-6, atol=1e-5)
    # sampled entries come from the same definition
    where = rng.integers(0, N * K, 40)
    assert np.array_equal(oracle.dw_linear_at(vals, mask, dY, M, K, N, where), dW.reshape(-1)[where])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [
    # Nb, Ci, H, W, Co, k, stride, pad
    (3, 5, 9, 9, 7, 3, 1, 1),
    (2, 4, 10, 8, 6, 3, 2, 1),
    (2, 3, 11, 11, 4, 7, 2, 3),
    (3, 6, 6, 6, 5, 1, 1, 0),
    (2, 6, 8, 8, 5, 1, 2, 0),
    (2, 2, 7, 9, 3, 5, 1, 2),
])
def test_conv_matches_library_weight_gradient(dtype, shape):
    Nb, Ci, H, W, Co, k, st, pad = shape
    rng = np.random.default_rng(sum(shape))
    OH, OW = (H + 2 * pad - k) // st + 1, (W + 2 * pad - k) // st + 1
    A = rng.standard_normal((Nb, Ci, H, W)).astype(np.float32)
    dY = rng.standard_normal((Nb, Co, OH, OW)).astype(np.float32)
    if dtype == "bf16":
        A, dY = _bf16(A), _bf16(dY)
    for r in (0.0, 0.6):
        vals, mask, Ad = _dense_pruned(A, 64, r)
        dW = oracle.dw_conv2d(vals, mask, dY, Nb, Ci, H, W, Co, k, k, st, pad)
        ref = torch.nn.grad.conv2d_weight(torch.from_numpy(Ad.reshape(Nb, Ci, H, W)), (Co, Ci, k, k),
                                          torch.from_numpy(_f64(dY).reshape(Nb, Co, OH, OW)), stride=st, padding=pad)
        assert np.allclose(dW, ref.numpy(), rtol=1e-6, atol=1e-6)
        where = rng.integers(0, dW.size, 25)
        assert np.array_equal(oracle.dw_conv2d_at(vals, mask, dY, Nb, Ci, H, W, Co, k, k, st, pad, where),
                              dW.reshape(-1)[where])
    vals, mask, _, _ = oracle.prune_pack(A, 64, 1.0)
    assert not oracle.dw_conv2d(vals, mask, dY, Nb, Ci, H, W, Co, k, k, st, pad).any()


def test_conv_1x1_equals_linear_over_pixels():
    rng = np.random.default_rng(4)
    Nb, Ci, H, W, Co = 3, 8, 5, 6, 7
    A = rng.standard_normal((Nb, Ci, H, W)).astype(np.float32)
    dY = rng.standard_normal((Nb, Co, H, W)).astype(np.float32)
    vals, mask, _, _ = oracle.prune_pack(A, 32, 0.5)
    dWc = oracle.dw_conv2d(vals, mask, dY, Nb, Ci, H, W, Co, 1, 1, 1, 0).reshape(Co, Ci)
    # the same pruned activation seen as [pixels, Ci] with the same dropped positions
    dense = oracle.unpack(vals, mask, A.size).reshape(Nb, Ci, H, W)
    A_rows = np.ascontiguousarray(dense.transpose(0, 2, 3, 1).reshape(-1, Ci))
    dY_rows = np.ascontiguousarray(dY.transpose(0, 2, 3, 1).reshape(-1, Co))
    v2, m2, _, _ = oracle.prune_pack(A_rows, A_rows.size, 0.0)
    dWl = oracle.dw_linear(v2, m2, dY_rows, A_rows.shape[0], Ci, Co)
    assert np.allclose(dWc, dWl, rtol=1e-6, atol=1e-6)


def test_grad_importance_closed_forms():
    assert oracle.grad_importance(np.full(1000, -2.5, np.float32)) == pytest.approx(2.5, rel=1e-7)
    one_hot = np.zeros(4096, np.float32)
    one_hot[17] = 1.0
    assert oracle.grad_importance(one_hot) == pytest.approx(1 / 64, rel=1e-7)
    rng = np.random.default_rng(9)
    w = rng.standard_normal(12345).astype(np.float32)
    ref = np.linalg.norm(w.astype(np.float64)) / np.sqrt(w.size)  # ||.||_F / sqrt(numel)
    assert oracle.grad_importance(w) == pytest.approx(ref, rel=1e-7)
    assert oracle.grad_importance(-3 * w) == pytest.approx(3 * ref, rel=1e-6)  # scale equivariance
    assert oracle.grad_importance(np.zeros(0, np.float32)) == 0.0
    assert oracle.grad_importance(np.zeros(10, np.float32)) == 0.0
