"""Pins for the oracle's activation gradient (Eq. 2, first line), gradient step (Alg. 1 line 14), normalisation-layer
gradients and grouped-convolution weight gradient -- CPU only.

None of these re-types the oracle's loops: they compare with library routines in float64 (numpy matmul,
torch.nn.grad.conv2d_input / conv2d_weight, autograd), with exact rational arithmetic for the bfloat16 rounding,
with the adjoint identity that ties dA and dW to the forward convolution, and with closed forms.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle


def _bf16(x):
    return torch.from_numpy(np.asarray(x, dtype=np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def _f64(a):
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def _nearest_bf16_bits(x: Fraction) -> int:
    """Exact round-to-nearest-even of a rational onto the bfloat16 grid (finite, normal range), by integer arithmetic."""
    if x == 0:
        return 0
    sign = 0x8000 if x < 0 else 0
    x = abs(x)
    e = 0
    while x >= 2:
        x /= 2
        e += 1
    while x < 1:
        x *= 2
        e -= 1
    scaled = x * 128  # 8 significant bits: 128 <= scaled < 256
    q, rem = divmod(scaled.numerator, scaled.denominator)
    twice = 2 * rem
    if twice > scaled.denominator or (twice == scaled.denominator and q % 2 == 1):
        q += 1
    if q == 256:
        q, e = 128, e + 1
    assert -126 <= e <= 127
    return sign | ((e + 127) << 7) | (q - 128)


def test_bf16_outputs_round_once_to_nearest_even():
    """dA of a 1-term contraction is one exact product of two bfloat16 numbers: the stored result must be that product
    rounded ONCE to nearest-even (going through float first would round twice)."""
    rng = np.random.default_rng(0)
    a = _bf16(rng.standard_normal(4000) * 3)
    w = _bf16(rng.standard_normal(4000) * 0.7)
    # tie cases: 1.0078125 * 1.5 = 1.51171875, halfway between two bfloat16 values, and friends
    a[:4] = _bf16([1.0078125, 1.0234375, -1.0078125, 3.0])
    w[:4] = _bf16([1.5, 1.5, 1.5, 0.33203125])
    for i in range(a.size):
        got = oracle.da_linear(a[i:i + 1], w[i:i + 1], 1, 1, 1)[0, 0]
        exact = Fraction(float(_f64(a[i:i + 1])[0])) * Fraction(float(_f64(w[i:i + 1])[0]))
        assert int(got) == _nearest_bf16_bits(exact), i


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_da_linear_is_matmul(dtype):
    rng = np.random.default_rng(1)
    M, K, N = 23, 31, 17  # all different: a transposed operand or output fails
    dY = rng.standard_normal((M, N)).astype(np.float32)
    W = rng.standard_normal((N, K)).astype(np.float32)
    if dtype == "bf16":
        dY, W = _bf16(dY), _bf16(W)
    dA = oracle.da_linear(dY, W, M, K, N)
    ref = _f64(dY) @ _f64(W)
    assert dA.shape == (M, K)
    tol = 1e-6 if dtype == "f32" else 2.0 ** -8
    assert np.allclose(_f64(dA), ref, rtol=tol, atol=1e-6)
    where = rng.integers(0, M * K, 50)
    assert np.array_equal(oracle.da_linear_at(dY, W, M, K, N, where), dA.reshape(-1)[where])


CONV_CASES = [
    # Nb, Ci, H, W, Co, kh, kw, stride, pad
    (2, 3, 9, 11, 4, 3, 3, 1, 1), (2, 5, 8, 8, 3, 3, 3, 2, 1), (1, 2, 7, 9, 6, 1, 1, 1, 0), (2, 4, 10, 8, 3, 1, 1, 2, 0),
    (1, 3, 12, 13, 2, 5, 5, 2, 2), (2, 2, 15, 15, 3, 7, 7, 2, 3), (1, 3, 6, 7, 2, 3, 3, 1, 0), (2, 3, 9, 9, 2, 3, 3, 3, 1),
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_da_conv2d_is_the_library_input_gradient(case):
    Nb, Ci, H, W, Co, kh, kw, st, pad = case
    rng = np.random.default_rng(sum(case))
    OH, OW = (H + 2 * pad - kh) // st + 1, (W + 2 * pad - kw) // st + 1
    dY = rng.standard_normal((Nb, Co, OH, OW)).astype(np.float32)
    Wt = rng.standard_normal((Co, Ci, kh, kw)).astype(np.float32)
    dA = oracle.da_conv2d(dY, Wt, Nb, Ci, H, W, Co, kh, kw, st, pad)
    ref = torch.nn.grad.conv2d_input((Nb, Ci, H, W), torch.from_numpy(Wt).double(), torch.from_numpy(dY).double(),
                                     stride=st, padding=pad).numpy()
    assert dA.shape == ref.shape
    assert np.allclose(dA, ref, rtol=1e-6, atol=1e-6)
    where = rng.integers(0, dA.size, 60)
    assert np.array_equal(oracle.da_conv2d_at(dY, Wt, Nb, Ci, H, W, Co, kh, kw, st, pad, where), dA.reshape(-1)[where])


@pytest.mark.parametrize("case", CONV_CASES[:5])
def test_adjoint_identity_ties_da_and_dw_to_the_forward_convolution(case):
    """<dY, conv(A, W)> = <dA, A> = <dW, W>: one scalar computed three ways, two of them by the oracle."""
    Nb, Ci, H, W, Co, kh, kw, st, pad = case
    rng = np.random.default_rng(7 + sum(case))
    OH, OW = (H + 2 * pad - kh) // st + 1, (W + 2 * pad - kw) // st + 1
    A = rng.standard_normal((Nb, Ci, H, W)).astype(np.float32)
    dY = rng.standard_normal((Nb, Co, OH, OW)).astype(np.float32)
    Wt = rng.standard_normal((Co, Ci, kh, kw)).astype(np.float32)
    Y = torch.nn.functional.conv2d(torch.from_numpy(A).double(), torch.from_numpy(Wt).double(), stride=st, padding=pad)
    lhs = float((Y.numpy() * dY.astype(np.float64)).sum())
    dA = oracle.da_conv2d(dY, Wt, Nb, Ci, H, W, Co, kh, kw, st, pad)
    vals, mask, _, _ = oracle.prune_pack(A.reshape(-1), A.size, 0.0)
    dW = oracle.dw_conv2d(vals, mask, dY, Nb, Ci, H, W, Co, kh, kw, st, pad)
    scale = float(np.abs(Y.numpy()).sum())
    assert abs(float((dA.astype(np.float64) * A).sum()) - lhs) <= 1e-5 * scale
    assert abs(float((dW.astype(np.float64) * Wt).sum()) - lhs) <= 1e-5 * scale


GROUPED_CASES = [
    # Nb, Ci, H, W, Co, kh, kw, stride, pad, groups
    (2, 6, 9, 8, 4, 3, 3, 1, 1, 2), (1, 8, 7, 7, 8, 3, 3, 1, 1, 8), (2, 4, 10, 9, 12, 3, 3, 2, 1, 4), (1, 6, 8, 8, 6, 5, 5, 2, 2, 3),
    (2, 4, 6, 6, 8, 1, 1, 1, 0, 2),
]


@pytest.mark.parametrize("case", GROUPED_CASES)
def test_grouped_da_is_the_library_input_gradient_and_satisfies_the_adjoint_identity(case):
    """Pins of the grouped activation gradient: the float64 library routine with `groups`; groups = 1 gives the plain
    oracle back; <dA, A> = <dW, W> with the grouped weight gradient of the oracle."""
    Nb, Ci, H, W, Co, kh, kw, st, pad, groups = case
    rng = np.random.default_rng(11 + sum(case))
    OH, OW = (H + 2 * pad - kh) // st + 1, (W + 2 * pad - kw) // st + 1
    A = rng.standard_normal((Nb, Ci, H, W)).astype(np.float32)
    dY = rng.standard_normal((Nb, Co, OH, OW)).astype(np.float32)
    Wt = rng.standard_normal((Co, Ci // groups, kh, kw)).astype(np.float32)
    dA = oracle.da_conv2d_grouped(dY, Wt, Nb, Ci, H, W, Co, kh, kw, st, pad, groups)
    ref = torch.nn.grad.conv2d_input((Nb, Ci, H, W), torch.from_numpy(Wt).double(), torch.from_numpy(dY).double(),
                                     stride=st, padding=pad, groups=groups).numpy()
    assert dA.shape == ref.shape
    assert np.allclose(dA, ref, rtol=1e-6, atol=1e-6)
    vals, mask, _, _ = oracle.prune_pack(A.reshape(-1), A.size, 0.0)
    dW = oracle.dw_conv2d_grouped(vals, mask, dY, Nb, Ci, H, W, Co, kh, kw, st, pad, groups)
    lhs = float((dA.astype(np.float64) * A).sum())
    assert abs(float((dW.astype(np.float64) * Wt).sum()) - lhs) <= 1e-5 * float(np.abs(dA.astype(np.float64) * A).sum())
    # one group: the plain routine, bit for bit
    W1 = rng.standard_normal((Co, Ci, kh, kw)).astype(np.float32)
    assert np.array_equal(oracle.da_conv2d_grouped(dY, W1, Nb, Ci, H, W, Co, kh, kw, st, pad, 1),
                          oracle.da_conv2d(dY, W1, Nb, Ci, H, W, Co, kh, kw, st, pad))


def test_one_by_one_convolution_input_gradient_is_the_linear_one():
    rng = np.random.default_rng(3)
    Nb, Ci, H, W, Co = 2, 5, 4, 3, 7
    dY = rng.standard_normal((Nb, Co, H, W)).astype(np.float32)
    Wt = rng.standard_normal((Co, Ci, 1, 1)).astype(np.float32)
    dA = oracle.da_conv2d(dY, Wt, Nb, Ci, H, W, Co, 1, 1, 1, 0)
    rows = np.ascontiguousarray(dY.transpose(0, 2, 3, 1).reshape(-1, Co))  # pixels as tokens
    lin = oracle.da_linear(rows, Wt.reshape(Co, Ci), rows.shape[0], Ci, Co)
    assert np.array_equal(lin.reshape(Nb, H, W, Ci).transpose(0, 3, 1, 2), dA)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_weight_update_closed_forms(dtype):
    rng = np.random.default_rng(4)
    W = rng.standard_normal(1000).astype(np.float32)
    dW = rng.standard_normal(1000).astype(np.float32)
    Wd = _bf16(W) if dtype == "bf16" else W
    assert np.array_equal(oracle.weight_update(Wd, dW, 0.0), Wd)                    # no step
    assert np.array_equal(oracle.weight_update(Wd, np.zeros_like(dW), 0.3), Wd)     # no gradient
    zero = np.zeros_like(Wd)
    got = oracle.weight_update(zero, dW, 1.0)                                        # W = 0, lr = 1: minus the gradient
    if dtype == "f32":
        assert np.array_equal(got, -dW)
    else:
        assert np.array_equal(got, _bf16(-dW))  # float -> bfloat16 of an exact float is a single rounding
    # the step moves against the gradient by lr * dW (checked in exact arithmetic on a few entries)
    lr = np.float32(0.0123)
    got = oracle.weight_update(Wd, dW, lr)
    for j in range(0, 1000, 97):
        exact = Fraction(float(_f64(Wd[j:j + 1])[0])) - Fraction(float(lr)) * Fraction(float(dW[j]))
        if dtype == "bf16":
            assert int(got[j]) == _nearest_bf16_bits(exact)
        else:
            assert abs(Fraction(float(got[j])) - exact) <= Fraction(float(np.spacing(np.abs(got[j])))) / 2


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("outer,C,inner", [(4, 5, 6), (7, 3, 1), (1, 8, 9), (3, 1, 10)])
def test_affine_grad_matches_autograd_and_closed_forms(dtype, outer, C, inner):
    rng = np.random.default_rng(outer * 100 + C * 10 + inner)
    x = rng.standard_normal((outer, C, inner)).astype(np.float32)
    dY = rng.standard_normal((outer, C, inner)).astype(np.float32)
    if dtype == "bf16":
        x, dY = _bf16(x), _bf16(dY)
    n = outer * C * inner
    for r in (0.0, 0.6):
        vals, mask, _, _ = oracle.prune_pack(x.reshape(-1), n, r)
        xhat = torch.from_numpy(_f64(oracle.unpack(vals, mask, n)).reshape(outer, C, inner))
        gamma = torch.ones(C, dtype=torch.float64, requires_grad=True)
        beta = torch.zeros(C, dtype=torch.float64, requires_grad=True)
        y = gamma.view(1, C, 1) * xhat + beta.view(1, C, 1)
        (y * torch.from_numpy(_f64(dY).reshape(outer, C, inner))).sum().backward()
        dgamma, dbeta = oracle.affine_grad(vals, mask, dY, outer, C, inner)
        assert np.allclose(dgamma, gamma.grad.numpy(), rtol=1e-6, atol=1e-6)
        assert np.allclose(dbeta, beta.grad.numpy(), rtol=1e-6, atol=1e-6)
    # dY = 1: dbeta counts the elements of a channel, dgamma sums the kept activations; ratio 1: dgamma = 0
    ones = np.ones((outer, C, inner), np.float32)
    ones = _bf16(ones) if dtype == "bf16" else ones
    vals, mask, _, _ = oracle.prune_pack(x.reshape(-1), n, 0.5)
    dgamma, dbeta = oracle.affine_grad(vals, mask, ones, outer, C, inner)
    assert np.array_equal(dbeta, np.full(C, outer * inner, np.float32))
    kept = _f64(oracle.unpack(vals, mask, n)).reshape(outer, C, inner)
    assert np.allclose(dgamma, kept.sum(axis=(0, 2)), rtol=1e-6, atol=1e-6)
    vals, mask, _, _ = oracle.prune_pack(x.reshape(-1), n, 1.0)
    assert not oracle.affine_grad(vals, mask, dY, outer, C, inner)[0].any()


GROUPED_CASES = [
    # Nb, Ci, H, W, Co, k, stride, pad, groups
    (2, 8, 9, 9, 12, 3, 1, 1, 4), (2, 6, 8, 10, 6, 3, 1, 1, 6), (1, 6, 11, 11, 6, 3, 2, 1, 6), (2, 4, 7, 7, 8, 1, 1, 0, 2),
    (2, 8, 8, 8, 8, 3, 1, 1, 1), (1, 4, 12, 12, 8, 5, 2, 2, 4),
]


@pytest.mark.parametrize("case", GROUPED_CASES)
def test_grouped_conv_weight_gradient_is_the_library_one(case):
    Nb, Ci, H, W, Co, k, st, pad, groups = case
    rng = np.random.default_rng(sum(case))
    OH, OW = (H + 2 * pad - k) // st + 1, (W + 2 * pad - k) // st + 1
    A = np.maximum(rng.standard_normal((Nb, Ci, H, W)), 0).astype(np.float32)
    dY = rng.standard_normal((Nb, Co, OH, OW)).astype(np.float32)
    for r in (0.0, 0.5):
        vals, mask, _, _ = oracle.prune_pack(A.reshape(-1), 64, r)
        dense = torch.from_numpy(oracle.unpack(vals, mask, A.size).reshape(A.shape)).double()
        ref = torch.nn.grad.conv2d_weight(dense, (Co, Ci // groups, k, k), torch.from_numpy(dY).double(), stride=st,
                                          padding=pad, groups=groups).numpy()
        dW = oracle.dw_conv2d_grouped(vals, mask, dY, Nb, Ci, H, W, Co, k, k, st, pad, groups)
        assert dW.shape == ref.shape
        assert np.allclose(dW, ref, rtol=1e-6, atol=1e-6)
        where = rng.integers(0, dW.size, 40)
        assert np.array_equal(oracle.dw_conv2d_grouped_at(vals, mask, dY, Nb, Ci, H, W, Co, k, k, st, pad, groups, where),
                              dW.reshape(-1)[where])
        if groups == 1:
            assert np.array_equal(dW, oracle.dw_conv2d(vals, mask, dY, Nb, Ci, H, W, Co, k, k, st, pad))
