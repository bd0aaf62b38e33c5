"""GPU parity: every entry point of the C ABI against the CPU oracle on the same seeded inputs.

Bars: masks, values, indices and counts bit-exact; dW and Gradient Importance within rel-L2 1e-5 for fp32
inputs and 2e-2 for bf16 inputs (the kernels accumulate exact bf16 products in fp32, so they sit far below it).
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_20354_amd as surgeon
import surgeon_workloads as wl
from parity_bars import TOL, assert_dw_close, rel_l2

pytestmark = pytest.mark.gpu

DEV = "cuda:0"

def host_bits(t):
    return wl.to_numpy_bits(t)


def draw(shape, dist, dtype, seed):
    if dist == "few":  # a handful of distinct magnitudes: almost everything ties
        g = torch.Generator().manual_seed(seed)
        t = torch.randint(-3, 4, shape, generator=g).to(torch.float32) * 0.5
        return t.to(torch.float32 if dtype == "f32" else torch.bfloat16)
    if dist == "const":
        return torch.full(shape, -1.25, dtype=torch.float32 if dtype == "f32" else torch.bfloat16)
    return wl.draw(shape, dist, dtype, seed)


def check_pack(A, g, r, want_idx=True, tag=""):
    print("prune_pack", tag, tuple(A.shape), A.dtype, "g=%d r=%g" % (g, r), flush=True)
    p = surgeon.prune_pack(A.to(DEV), g, r, want_idx=want_idx)
    torch.cuda.synchronize()
    o_vals, o_mask, o_idx, o_k = oracle.prune_pack(host_bits(A).reshape(-1), g, r)
    assert p.k_total == o_k
    assert np.array_equal(p.mask.cpu().numpy().view(np.uint64), o_mask), "mask"
    got_vals = host_bits(p.vals)
    assert np.array_equal(got_vals.view(np.uint8), o_vals.view(np.uint8)), "vals"
    if want_idx:
        assert np.array_equal(p.idx.cpu().numpy().view(np.uint32), o_idx), "idx"
    return p, (o_vals, o_mask)


# ------------------------------------------------------------------------------------------------
# Gradient Importance (Eq. 4)
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n", [0, 1, 5, 255, 4096, 4097, 65539, 1_000_003, 5_000_000])
def test_grad_importance(n):
    print("grad_importance n =", n, flush=True)
    x = wl.draw((n,), "normal", "f32", 100 + n % 97) * 3.0
    got = surgeon.grad_importance(x.to(DEV)).item()
    ref = oracle.grad_importance(x.numpy())
    assert abs(got - ref) <= 1e-5 * max(ref, 1e-30)
    if n > 8:  # a view that is only 4-byte aligned takes the scalar-load kernel
        got = surgeon.grad_importance(x.to(DEV)[1:]).item()
        ref = oracle.grad_importance(x.numpy()[1:])
        assert abs(got - ref) <= 1e-5 * ref


@pytest.mark.parametrize("n_layers", [1, 3, 28, 70, 266])
def test_grad_importance_batched(n_layers):
    """One call for all layers (also more than 64, which takes several launches) against the oracle per layer."""
    rng = np.random.default_rng(n_layers)
    sizes = [int(s) for s in rng.choice([0, 1, 7, 432, 4096, 16384, 16385, 51200, 230400, 1_000_003], n_layers)]
    sizes[0] = 1_000_003
    layers = [wl.draw((s,), "normal", "f32", 1000 + i) * (1.0 + i % 5) for i, s in enumerate(sizes)]
    dev_layers = [x.to(DEV) for x in layers]
    if n_layers >= 3:
        dev_layers[2] = torch.cat([torch.zeros(1, device=DEV), dev_layers[2]])[1:]  # one pointer only 4-byte aligned
    G = torch.full((n_layers,), -1.0, device=DEV)
    ws = torch.empty(surgeon.surgeon_grad_importance_batched_ws_bytes(dev_layers), dtype=torch.uint8, device=DEV)
    surgeon.surgeon_grad_importance_batched(dev_layers, G, ws)
    got = G.cpu().numpy()
    for i, x in enumerate(layers):
        ref = oracle.grad_importance(x.numpy())
        assert abs(got[i] - ref) <= 1e-5 * max(ref, 1e-30), (i, sizes[i])


def test_grad_importance_closed_forms():
    c = torch.full((123457,), -2.5, device=DEV)
    assert surgeon.grad_importance(c).item() == pytest.approx(2.5, rel=1e-6)
    one_hot = torch.zeros(1 << 20, device=DEV)
    one_hot[12345] = 1.0
    assert surgeon.grad_importance(one_hot).item() == pytest.approx(2.0 ** -10, rel=1e-6)


# ------------------------------------------------------------------------------------------------
# prune + pack (Alg. 1 lines 6-7): the three selection paths
# ------------------------------------------------------------------------------------------------
REG_CASES = [(32768, 512), (4096 * 5 + 1000, 4096), (768 * 50, 768), (3072 * 9, 3072), (64 * 100, 64),
             (128 * 33 + 64, 128), (320 * 20, 320), (1280 * 7 + 5, 1280), (2048 * 3, 2048), (4096, 4096), (64, 64)]
MEM_CASES = [(1000, 100), (5000, 1000), (777, 777), (4095 * 3, 4095), (10, 3), (130, 65), (1, 1), (63, 63)]
GLOBAL_CASES = [(100000, 100000), (300000, 50000), (20000, 5000), (1 << 20, 1 << 20), (70001, 70001), (12345, 4097)]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n,g", REG_CASES + MEM_CASES + GLOBAL_CASES)
def test_prune_pack_matches_oracle(dtype, n, g):
    seed = n * 7 + g
    for dist in ("normal", "relu", "few"):
        for r in (0.0, 0.3, 0.5, 0.9, 0.95, 1.0):
            A = draw((n,), dist, dtype, seed)
            check_pack(A, g, r, want_idx=(r != 0.3), tag=dist)
    check_pack(draw((n,), "const", dtype, seed), g, 0.7, tag="const")


TWO_READ_CASES = [(100000, 100000), (300000, 50000), (1 << 20, 1 << 20), (70001, 70001), (32768 * 3 + 10, 32768),
                  (40000 * 7 + 33000, 40000)]


@pytest.mark.parametrize("margin", [5.0, 0.3, -1.0])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_prune_pack_long_groups_two_reads(dtype, margin):
    """Groups of 32768 elements or more: the sampled bracket (default margin), a narrow bracket that often misses the
    threshold, and a negative margin under which every group takes the full-width route; all three bit-exact."""
    surgeon.surgeon_set_select_margin(margin)
    try:
        for n, g in TWO_READ_CASES:
            seed = n * 3 + g
            for dist in ("normal", "relu", "few", "image01"):
                for r in (0.0, 0.3, 0.5, 0.9, 0.999, 1.0):
                    check_pack(draw((n,), dist, dtype, seed), g, r, want_idx=(r == 0.5), tag="%s m=%g" % (dist, margin))
            check_pack(draw((n,), "const", dtype, seed), g, 0.7, tag="const")
        # plateaus at the top and inside the populated range (a clipped activation), negative zeros, non-finite values
        a = torch.randn(200000).clamp_(-1.0, 1.0)
        a[::7] = -0.0
        a[5], a[70000], a[150001] = float("inf"), float("nan"), float("-inf")
        for r in (0.2, 0.5, 0.7, 0.9):
            check_pack(a, 200000, r)
            check_pack(a.to(torch.bfloat16), 100000, r)
    finally:
        surgeon.surgeon_set_select_margin(5.0)


def test_prune_pack_signed_zero_and_non_finite():
    a = torch.zeros(4096)
    a[::3] = -0.0
    a[5], a[70], a[900], a[901] = float("inf"), float("-inf"), float("nan"), 1e38
    for g in (4096, 1000, 512):
        p, _ = check_pack(a, g, 0.9)
    A = a.clone()
    A[1000:3000] = torch.randn(2000)
    check_pack(A, 4096, 0.5)
    check_pack(A.to(torch.bfloat16), 4096, 0.5)


def test_prune_pack_empty_and_determinism():
    p = surgeon.prune_pack(torch.zeros(0, device=DEV), 64, 0.5)
    assert p.k_total == 0 and p.mask.numel() == 0
    A = wl.draw((4096 * 300 + 77,), "relu", "f32", 5).to(DEV)
    first = surgeon.prune_pack(A, 4096, 0.4, want_idx=True)
    with torch.cuda.stream(torch.cuda.Stream()):
        second = surgeon.prune_pack(A, 4096, 0.4, want_idx=True)
    torch.cuda.synchronize()
    assert torch.equal(first.mask, second.mask) and torch.equal(first.vals, second.vals)
    assert torch.equal(first.idx, second.idx)


# ------------------------------------------------------------------------------------------------
# dW from the packed activation (Eq. 2, Alg. 1 lines 11-12)
# ------------------------------------------------------------------------------------------------
def run_linear(M, K, N, dtype, r, g=None, seed=0):
    print("dw linear", (M, K, N), dtype, "r=%g" % r, flush=True)
    A = wl.draw((M, K), "normal", dtype, seed + 1)
    dY = wl.draw((M, N), "normal", dtype, seed + 2)
    p, (o_vals, o_mask) = check_pack(A, g or K, r, want_idx=False)
    desc = surgeon.linear_desc(M, K, N, surgeon.F32 if dtype == "f32" else surgeon.BF16, p.k_total)
    dW = surgeon.dw_from_packed(desc, p, dY.to(DEV))
    torch.cuda.synchronize()
    ref = oracle.dw_linear(o_vals, o_mask, host_bits(dY), M, K, N)
    return dW.cpu().numpy(), ref


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,K,N", [(64, 512, 256), (100, 70, 50), (300, 129, 257), (33, 64, 64), (1000, 768, 96),
                                   (1, 64, 64), (517, 320, 1280)])
def test_dw_linear(dtype, M, K, N):
    for r in (0.0, 0.5, 0.9):
        got, ref = run_linear(M, K, N, dtype, r, seed=M + K + N)
        assert got.shape == ref.shape == (N, K)
        assert_dw_close(got, ref, dtype)
    got, _ = run_linear(M, K, N, dtype, 1.0)
    assert not got.any()  # nothing cached: the gradient is exactly zero


@pytest.mark.parametrize("M,K,N", [(130, 136, 264), (1000, 768, 384), (77, 8, 8), (4096, 320, 1280), (257, 1032, 72),
                                   (2000, 768, 19), (333, 72, 1), (129, 264, 131)])
def test_dw_linear_bf16_matrix_core_path(M, K, N):
    """bf16 linears whose in-feature count is a multiple of 8 take the dense bf16-MFMA path; an out-feature count
    that is not (a 19-class head) reads dY element by element."""
    for r in (0.5, 0.93):
        got, ref = run_linear(M, K, N, "bf16", r, seed=3 * M + K)
        assert_dw_close(got, ref, "bf16")


def test_dw_linear_ratio0_is_dense_gradient():
    M, K, N = 200, 256, 192
    A = wl.draw((M, K), "normal", "f32", 11)
    dY = wl.draw((M, N), "normal", "f32", 12)
    p = surgeon.prune_pack(A.to(DEV), K, 0.0)
    dW = surgeon.dw_from_packed(surgeon.linear_desc(M, K, N, surgeon.F32, p.k_total), p, dY.to(DEV))
    dense = dY.double().T @ A.double()
    assert_dw_close(dW.cpu().numpy(), dense.numpy(), "f32")


def run_conv(shape, dtype, r, dist="relu", seed=0):
    Nb, Ci, H, W, Co, k, st = shape[:7]
    pad = shape[7] if len(shape) > 7 else k // 2
    print("dw conv", shape, dtype, "r=%g" % r, flush=True)
    OH, OW = (H + 2 * pad - k) // st + 1, (W + 2 * pad - k) // st + 1
    A = wl.draw((Nb, Ci, H, W), dist, dtype, seed + 1)
    dY = wl.draw((Nb, Co, OH, OW), "normal", dtype, seed + 2)
    p, (o_vals, o_mask) = check_pack(A, 4096, r, want_idx=False)
    desc = surgeon.conv2d_desc(Nb, Ci, H, W, Co, k, k, st, pad, surgeon.F32 if dtype == "f32" else surgeon.BF16, p.k_total)
    dW = surgeon.dw_from_packed(desc, p, dY.to(DEV))
    torch.cuda.synchronize()
    ref = oracle.dw_conv2d(o_vals, o_mask, host_bits(dY), Nb, Ci, H, W, Co, k, k, st, pad)
    return dW.cpu().numpy(), ref


CONV_SHAPES = [
    # Nb, Ci, H, W, Co, k, stride
    (4, 16, 32, 32, 160, 3, 1), (3, 160, 16, 16, 160, 3, 1), (2, 160, 32, 32, 320, 3, 2), (2, 16, 32, 32, 160, 1, 1),
    (2, 160, 32, 32, 320, 1, 2), (2, 3, 32, 32, 16, 3, 1), (2, 3, 64, 64, 64, 7, 2), (1, 3, 224, 224, 64, 7, 2),
    (2, 64, 56, 56, 64, 3, 1), (2, 64, 56, 56, 256, 1, 1), (2, 128, 56, 56, 128, 3, 2), (2, 512, 7, 7, 512, 3, 1),
    (2, 5, 9, 9, 7, 5, 1), (3, 6, 12, 12, 20, 3, 1), (2, 256, 14, 14, 1024, 1, 1), (2, 40, 13, 13, 24, 3, 1),
    (3, 64, 8, 8, 160, 3, 1), (2, 48, 24, 24, 32, 3, 2), (2, 33, 40, 40, 20, 3, 1),
    # 1x1 layers on maps whose pixel count 4 does not divide (they stay on the fp32 matrix cores: the bf16 route staged
    # element by element was measured no faster); the packed tensor then ends inside a mask word
    (2, 70, 7, 7, 130, 1, 1), (1, 3, 7, 7, 5, 1, 1), (3, 64, 9, 5, 64, 1, 1), (5, 512, 7, 7, 256, 1, 1), (2, 8, 5, 5, 8, 1, 1),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", CONV_SHAPES)
def test_dw_conv(dtype, shape):
    for r in (0.0, 0.7):
        got, ref = run_conv(shape, dtype, r, seed=sum(shape))
        assert got.shape == ref.shape
        assert_dw_close(got, ref, dtype, shape)
    got, _ = run_conv(shape, dtype, 1.0)
    assert not got.any()


# unpadded and strided filters: the patch kept in LDS is narrower than the input row
UNPADDED_SHAPES = [
    # Nb, Ci, H, W, Co, k, stride, pad
    (2, 5, 9, 14, 65, 7, 2, 0), (3, 1, 7, 8, 65, 3, 3, 0), (3, 1, 33, 32, 65, 3, 2, 0), (2, 16, 17, 17, 16, 3, 1, 0),
    (2, 33, 16, 16, 64, 1, 2, 0), (2, 8, 20, 20, 24, 5, 2, 1), (1, 64, 14, 14, 65, 3, 3, 1),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", UNPADDED_SHAPES)
def test_dw_conv_unpadded_and_strided(dtype, shape):
    for r in (0.0, 0.5):
        got, ref = run_conv(shape, dtype, r, seed=sum(shape))
        assert got.shape == ref.shape
        assert_dw_close(got, ref, dtype, shape)


# fp32 3x3 stride-1 pad-1 layers of width 8 / 16 / 32 with few kept elements: gradient from the kept elements alone
SPARSE_SHAPES = [
    # Nb, Ci, H, W, Co, k, stride
    (5, 160, 32, 32, 160, 3, 1), (3, 320, 16, 16, 320, 3, 1), (7, 640, 8, 8, 640, 3, 1), (2, 33, 12, 32, 70, 3, 1),
    (3, 5, 24, 16, 32, 3, 1), (9, 40, 16, 8, 129, 3, 1), (1, 1, 8, 8, 64, 3, 1), (2, 96, 4, 32, 33, 3, 1),
]


@pytest.mark.parametrize("shape", SPARSE_SHAPES)
def test_dw_conv_from_kept_elements_only(shape):
    Nb, Ci, H, W, Co = shape[:5]
    n = Nb * Ci * H * W
    # 0.8: 20 % kept, still this kernel where the input channels fill 64-channel workgroups (taps shared by channels)
    for r, dist in ((0.9, "relu"), (0.97, "normal"), (0.85, "normal"), (0.8, "relu")):
        k = surgeon.surgeon_packed_sizes(n, 4096, r, surgeon.F32)[0]
        desc = surgeon.conv2d_desc(Nb, Ci, H, W, Co, 3, 3, 1, 1, surgeon.F32, k)
        wide = -(-Ci // 64) * 64 <= -(-Ci // 32) * 32  # 64-channel workgroups pad the channels no more than 32-channel ones
        assert surgeon.surgeon_dw_kernel_class(desc) == ("dw_sparse" if r >= 0.85 or wide else "dw")
        got, ref = run_conv(shape, "f32", r, dist=dist, seed=sum(shape))
        assert got.shape == ref.shape
        assert_dw_close(got, ref, "f32", shape)
    # the same layer with more elements kept takes the dense kernel; both agree with the oracle, hence with each other
    k = surgeon.surgeon_packed_sizes(n, 4096, 0.5, surgeon.F32)[0]
    assert surgeon.surgeon_dw_kernel_class(surgeon.conv2d_desc(Nb, Ci, H, W, Co, 3, 3, 1, 1, surgeon.F32, k)) == "dw"


def test_dw_conv_from_kept_elements_is_deterministic_and_profiled():
    Nb, Ci, H, W, Co = 6, 64, 16, 16, 96
    A = wl.draw((Nb, Ci, H, W), "relu", "f32", 71).to(DEV)
    dY = wl.draw((Nb, Co, H, W), "normal", "f32", 72).to(DEV)
    p = surgeon.prune_pack(A, 4096, 0.9)
    desc = surgeon.conv2d_desc(Nb, Ci, H, W, Co, 3, 3, 1, 1, surgeon.F32, p.k_total)
    surgeon.surgeon_profile_begin()
    a = surgeon.dw_from_packed(desc, p, dY)
    b = surgeon.dw_from_packed(desc, p, dY)
    torch.cuda.synchronize()
    prof = surgeon.surgeon_profile_end()
    assert torch.equal(a, b)
    assert prof["dw_sparse"][1] == 2 and prof["dw"][1] == 0


def test_dw_group_hint_changes_nothing():
    """The optional (group_len, r) hint only selects a cheaper pre-pass: same bits with and without it."""
    Nb, Ci, H, W, Co = 4, 160, 32, 32, 160
    A = wl.draw((Nb, Ci, H, W), "relu", "f32", 21).to(DEV)
    dY = wl.draw((Nb, Co, H, W), "normal", "f32", 22).to(DEV)
    for g, r in ((4096, 0.45), (512, 0.9), (4096 * 3, 0.5)):  # the last one is not eligible for the closed form
        p = surgeon.prune_pack(A, g, r)
        plain = surgeon.conv2d_desc(Nb, Ci, H, W, Co, 3, 3, 1, 1, surgeon.F32, p.k_total)
        hinted = surgeon.conv2d_desc(Nb, Ci, H, W, Co, 3, 3, 1, 1, surgeon.F32, p.k_total, group_len=g, r=r)
        ws = torch.empty(surgeon.surgeon_dw_ws_bytes(plain), dtype=torch.uint8, device=DEV)
        a, b = torch.empty(Co, Ci, 3, 3, device=DEV), torch.empty(Co, Ci, 3, 3, device=DEV)
        surgeon.surgeon_dw_from_packed(plain, p.vals, p.mask, dY, a, ws)
        surgeon.surgeon_dw_from_packed(hinted, p.vals, p.mask, dY, b, ws)
        torch.cuda.synchronize()
        assert torch.equal(a, b)


@pytest.mark.parametrize("case", [("linear", 300, 320, 192, 320, 0.9), ("linear", 257, 768, 256, 768, 0.0),
                                  ("linear", 130, 3072, 128, 3072, 0.5), ("linear", 64, 4096, 64, 4096, 0.0),
                                  ("linear", 96, 4096, 72, 4096, 0.97), ("linear", 1003, 64, 64, 64, 0.5),
                                  ("linear", 333, 128, 96, 128, 0.9), ("linear", 257, 256, 64, 256, 0.0),
                                  ("linear", 130, 192, 64, 192, 0.7), ("conv1x1", 3, 70, 8, 96, 4096, 0.6),
                                  ("conv1x1", 5, 64, 12, 128, 4096, 0.0)])
def test_dw_bf16_dense_copy_with_and_without_the_hint(case):
    """bf16 linear and 1x1 layers rebuild the dense activation first; with the packing hint one wavefront per group
    expands its kept values from LDS (every group length up to 4096, groups of one to four mask words taken 64 words at a
    time, nothing dropped, nearly everything dropped, a ragged last group), without it the rank-table kernel does.  Same bits either way, and the oracle's dW."""
    print("dense copy", case, flush=True)
    if case[0] == "linear":
        _, M, K, N, g, r = case
        A = wl.draw((M, K), "normal", "bf16", 31)
        dY = wl.draw((M, N), "normal", "bf16", 32)
        p, (o_vals, o_mask) = check_pack(A, g, r, want_idx=False)
        plain = surgeon.linear_desc(M, K, N, surgeon.BF16, p.k_total)
        hinted = surgeon.linear_desc(M, K, N, surgeon.BF16, p.k_total, group_len=g, r=r)
        shape = (N, K)
        ref = oracle.dw_linear(o_vals, o_mask, host_bits(dY), M, K, N)
    else:
        _, Nb, Ci, HW, Co, g, r = case
        A = wl.draw((Nb, Ci, HW, HW), "relu", "bf16", 33)
        dY = wl.draw((Nb, Co, HW, HW), "normal", "bf16", 34)
        p, (o_vals, o_mask) = check_pack(A, g, r, want_idx=False)
        plain = surgeon.conv2d_desc(Nb, Ci, HW, HW, Co, 1, 1, 1, 0, surgeon.BF16, p.k_total)
        hinted = surgeon.conv2d_desc(Nb, Ci, HW, HW, Co, 1, 1, 1, 0, surgeon.BF16, p.k_total, group_len=g, r=r)
        shape = (Co, Ci, 1, 1)
        ref = oracle.dw_conv2d(o_vals, o_mask, host_bits(dY), Nb, Ci, HW, HW, Co, 1, 1, 1, 0)
    ws = torch.empty(max(surgeon.surgeon_dw_ws_bytes(plain), surgeon.surgeon_dw_ws_bytes(hinted)), dtype=torch.uint8, device=DEV)
    a, b = torch.empty(shape, device=DEV), torch.empty(shape, device=DEV)
    dYd = dY.to(DEV)
    surgeon.surgeon_dw_from_packed(plain, p.vals, p.mask, dYd, a, ws)
    surgeon.surgeon_dw_from_packed(hinted, p.vals, p.mask, dYd, b, ws)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    assert_dw_close(b.cpu().numpy(), ref, "bf16")


def test_dw_is_deterministic():
    shape = (8, 160, 32, 32, 160, 3, 1)
    Nb, Ci, H, W, Co, k, st = shape
    A = wl.draw((Nb, Ci, H, W), "relu", "f32", 1).to(DEV)
    dY = wl.draw((Nb, Co, H, W), "normal", "f32", 2).to(DEV)
    p = surgeon.prune_pack(A, 4096, 0.6)
    desc = surgeon.conv2d_desc(Nb, Ci, H, W, Co, k, k, st, 1, surgeon.F32, p.k_total)
    a = surgeon.dw_from_packed(desc, p, dY).clone()
    b = surgeon.dw_from_packed(desc, p, dY)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


# ------------------------------------------------------------------------------------------------
# the five workloads at reduced batch: the whole path per distinct layer shape
# ------------------------------------------------------------------------------------------------
def whole_path_layer(cfg, li, layer, r):
    """select + pack + dW + Gradient Importance for one layer; returns (G_gpu, G_oracle)."""
    A, dY = wl.layer_tensors(cfg, li, layer)
    p, (o_vals, o_mask) = check_pack(A, layer.group_len, r, want_idx=False, tag=layer.name)
    dt = surgeon.F32 if layer.dtype == "f32" else surgeon.BF16
    if layer.kind == "linear":
        desc = surgeon.linear_desc(layer.M, layer.K, layer.N, dt, p.k_total)
        ref = oracle.dw_linear(o_vals, o_mask, host_bits(dY), layer.M, layer.K, layer.N)
    else:
        desc = surgeon.conv2d_desc(layer.Nb, layer.Ci, layer.H, layer.W, layer.Co, layer.kh, layer.kw, layer.stride,
                                   layer.pad, dt, p.k_total)
        ref = oracle.dw_conv2d(o_vals, o_mask, host_bits(dY), layer.Nb, layer.Ci, layer.H, layer.W, layer.Co,
                               layer.kh, layer.kw, layer.stride, layer.pad)
    dW = surgeon.dw_from_packed(desc, p, dY.to(DEV))
    G = surgeon.grad_importance(dW)
    torch.cuda.synchronize()
    assert_dw_close(dW.cpu().numpy(), ref, layer.dtype, layer.name)
    o_G = oracle.grad_importance(ref)
    assert abs(G.item() - o_G) <= 1e-5 * max(o_G, 1e-30), layer.name
    return G.item(), o_G


@pytest.mark.parametrize("cfg,batch_div", [(0, 1), (1, 100), (2, 64), (3, 197), (4, 64)])
def test_workload_shapes_reduced(cfg, batch_div):
    layers = [wl.shrink(l, batch_div) for l in wl.distinct_shapes(wl.config_layers(cfg))]
    lo, hi = wl.RATIO_RANGE[cfg]
    # importance pass at the static ratio, then the ratio rule (Eq. 5-7), then the adaptation pass
    G_gpu, G_ref = [], []
    for li, layer in enumerate(layers):
        g, o = whole_path_layer(cfg, li, layer, wl.IMPORTANCE_PASS_RATIO if cfg else 0.5)
        G_gpu.append(g)
        G_ref.append(o)
    if cfg == 0:
        return
    m = [l.n * l.elem_bytes for l in layers]
    ratios = surgeon.surgeon_layer_ratios(G_gpu, m, lo, hi).numpy()
    assert np.allclose(ratios, oracle.layer_ratios(np.array(G_ref, np.float32), np.array(m, np.uint64), lo, hi), atol=1e-5)
    assert ratios.min() == pytest.approx(lo, abs=1e-6) and ratios.max() <= hi + 1e-6
    for li, layer in enumerate(layers):
        whole_path_layer(cfg, li, layer, float(ratios[li]))


# ------------------------------------------------------------------------------------------------
# all five workloads at FULL size, in the launch configuration the benchmark times: complete select/pack parity,
# dW on sampled entries evaluated one by one from the definition (the oracle cannot finish a full-size dW)
# ------------------------------------------------------------------------------------------------
def full_size_layer(cfg, name, r, n_samples=2048):
    layers = wl.config_layers(cfg)
    li = [l.name for l in layers].index(name)
    layer = layers[li]
    A, dY = wl.layer_tensors(cfg, li, layer)
    p, (o_vals, o_mask) = check_pack(A, layer.group_len, r, want_idx=False, tag="cfg%d %s" % (cfg, name))
    dt = surgeon.F32 if layer.dtype == "f32" else surgeon.BF16
    where = np.random.default_rng(1000 * cfg + li).integers(0, layer.n_w, n_samples)
    if layer.kind == "linear":
        desc = surgeon.linear_desc(layer.M, layer.K, layer.N, dt, p.k_total)
    else:
        desc = surgeon.conv2d_desc(layer.Nb, layer.Ci, layer.H, layer.W, layer.Co, layer.kh, layer.kw, layer.stride,
                                   layer.pad, dt, p.k_total)
    kernel_class = surgeon.surgeon_dw_kernel_class(desc)
    dW = surgeon.dw_from_packed(desc, p, dY.to(DEV))  # passes the packing's (group_len, r) on, as the benchmark does
    G = surgeon.grad_importance(dW)
    torch.cuda.synchronize()
    if layer.kind == "linear":
        ref = oracle.dw_linear_at(o_vals, o_mask, host_bits(dY), layer.M, layer.K, layer.N, where)
    else:
        ref = oracle.dw_conv2d_at(o_vals, o_mask, host_bits(dY), layer.Nb, layer.Ci, layer.H, layer.W, layer.Co,
                                  layer.kh, layer.kw, layer.stride, layer.pad, where)
    got = dW.cpu().numpy().reshape(-1)
    assert np.isfinite(got).all()
    assert_dw_close(got[where], ref, layer.dtype, (cfg, name, r))
    # Gradient Importance of the full gradient the GPU produced, against the oracle on the same values
    assert abs(G.item() - oracle.grad_importance(got)) <= 1e-5 * G.item()
    return kernel_class


# WideResNet-28-10, batch 200 (fp32).  0.9 is the importance pass; s3b2.conv2 at 0.79 is what the ratio rule gives
# the last stage: the 16-wavefront kept-elements kernel with shared taps on 640 channels.
@pytest.mark.parametrize("name,r", [("s1b2.conv1", 0.9), ("s2b1.conv1", 0.45), ("s3b2.conv2", 0.3), ("s2b1.shortcut", 0.6),
                                    ("stem", 0.5), ("s3b2.conv2", 0.79), ("s3b3.conv1", 0.9), ("s2b3.conv2", 0.9),
                                    ("s3b1.conv1", 0.9), ("s1b1.shortcut", 0.9)])
def test_benchmark_workload_full_size_sampled(name, r):
    cls = full_size_layer(1, name, r)
    if name in ("s3b2.conv2", "s3b3.conv1", "s2b3.conv2", "s1b2.conv1") and r >= 0.79:
        assert cls == "dw_sparse"


# ResNet-50, batch 64 (bf16, post-ReLU): the stem, a 3x3 and a 1x1 of each stage, both kinds of downsample
@pytest.mark.parametrize("name,r", [("stem", 0.5), ("s1b1.conv2", 0.9), ("s2b1.conv2", 0.7), ("s3b2.conv2", 0.9),
                                    ("s4b2.conv2", 0.6), ("s1b1.conv1", 0.9), ("s1b1.conv3", 0.8), ("s2b2.conv1", 0.9),
                                    ("s3b2.conv3", 0.55), ("s4b2.conv1", 0.9), ("s4b3.conv3", 0.95),
                                    ("s1b1.downsample", 0.9), ("s2b1.downsample", 0.75), ("s4b1.downsample", 0.9)])
def test_resnet50_workload_full_size_sampled(name, r):
    full_size_layer(2, name, r)


# ViT-B/16, 12 608 tokens (bf16): the wide tile and the long split contraction are only reached at this size
@pytest.mark.parametrize("name,r", [("blk0.qkv", 0.9), ("blk0.qkv", 0.6), ("blk3.proj", 0.9), ("blk3.proj", 0.5),
                                    ("blk5.fc1", 0.9), ("blk5.fc1", 0.7), ("blk11.fc2", 0.9), ("blk11.fc2", 0.55)])
def test_vit_workload_full_size_sampled(name, r):
    full_size_layer(3, name, r)


# segmentation transformer, batch 2 (bf16): 65 536-token layers of 64 channels, the reduced-token kv layer, the
# 3072 -> 768 fuse layer (201 M elements) and the 19-class head (dY rows not 16-byte aligned)
@pytest.mark.parametrize("name,r", [("st1b1.fc1", 0.9), ("st1b1.q", 0.8), ("st1b2.fc2", 0.9), ("st2b1.proj", 0.7),
                                    ("st3b1.kv", 0.9), ("st3b7.fc2", 0.75), ("st4b1.fc1", 0.9), ("dec.proj1", 0.9),
                                    ("dec.fuse", 0.9), ("dec.fuse", 0.65), ("dec.cls", 0.9), ("dec.cls", 0.6)])
def test_segmentation_workload_full_size_sampled(name, r):
    full_size_layer(4, name, r)


# ------------------------------------------------------------------------------------------------
# many tensors in one call
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_prune_pack_batched_matches_single_calls_and_oracle(dtype):
    """70 tensors of mixed group lengths, sizes and ratios (more than one batch of 48, every kernel variant, ragged last
    groups, a ratio of 1): the batched call writes the same bits as one call per tensor, which match the oracle."""
    rng = np.random.default_rng(5)
    g_choices = [64, 128, 256, 320, 512, 768, 1280, 2048, 3072, 4096, 4096, 4096]
    As, gs, rs = [], [], []
    for i in range(70):
        g = int(rng.choice(g_choices))
        n = g * int(rng.integers(1, 40)) + (int(rng.integers(0, g // 64)) * 64 if i % 3 == 0 else 0)
        As.append(wl.draw((n,), "relu" if i % 2 else "normal", dtype, 9000 + i))
        gs.append(g)
        rs.append(1.0 if i == 7 else float(rng.choice([0.0, 0.3, 0.5, 0.9, 0.95])))
    dev_A = [a.to(DEV) for a in As]
    vals, masks = [], []
    for a, g, r in zip(dev_A, gs, rs):
        k = surgeon.surgeon_packed_sizes(a.numel(), g, r, surgeon.F32 if dtype == "f32" else surgeon.BF16)[0]
        vals.append(torch.full((max(k, 1),), 7.0, dtype=a.dtype, device=DEV))
        masks.append(torch.full(((a.numel() + 63) // 64,), -1, dtype=torch.int64, device=DEV))
    surgeon.surgeon_prune_pack_batched(dev_A, gs, rs, vals, masks)
    torch.cuda.synchronize()
    for i, (a, g, r) in enumerate(zip(As, gs, rs)):
        o_vals, o_mask, _, o_k = oracle.prune_pack(host_bits(a), g, r)
        assert np.array_equal(masks[i].cpu().numpy().view(np.uint64), o_mask), (i, g, r)
        assert np.array_equal(host_bits(vals[i])[:o_k].view(np.uint8), o_vals.view(np.uint8)), (i, g, r)
        single = surgeon.prune_pack(dev_A[i], g, r)
        assert torch.equal(single.mask, masks[i]) and torch.equal(single.vals, vals[i][:o_k])
    # a tensor that does not take the in-register path is refused before anything is launched
    with pytest.raises(surgeon.SurgeonError) as e:
        surgeon.surgeon_prune_pack_batched([dev_A[0], dev_A[1]], [gs[0], 100], [0.5, 0.5], vals[:2], masks[:2])
    assert e.value.status == 3


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_select_pack_pattern_probe_keeps_what_its_threshold_says(dtype):
    """The benchmark aid does what its header says: mask bit = magnitude bits >= threshold, the kept values of a group in
    index order at group * k_cap, at most k_cap of them."""
    n, k_cap = 5 * 4096, 700
    A = wl.draw((n,), "normal", dtype, 77)
    as_uint = (lambda t: host_bits(t).view(np.uint32)) if dtype == "f32" else (lambda t: host_bits(t).view(np.uint16))
    bits = as_uint(A)
    thr = 0.9
    thr_bits = int(as_uint(torch.tensor([thr], dtype=A.dtype))[0])
    vals = torch.zeros(5 * k_cap, dtype=A.dtype, device=DEV)
    mask = torch.zeros(n // 64, dtype=torch.int64, device=DEV)
    surgeon.surgeon_select_pack_pattern_probe(A.to(DEV), thr_bits, k_cap, vals, mask)
    torch.cuda.synchronize()
    mag = bits & (0x7fffffff if dtype == "f32" else 0x7fff)
    keep = mag >= thr_bits
    want_mask = np.packbits(keep.reshape(-1, 64), axis=1, bitorder="little").view(np.uint64).reshape(-1)
    assert np.array_equal(mask.cpu().numpy().view(np.uint64), want_mask)
    got = as_uint(vals.cpu())
    for g in range(5):
        kept = bits[g * 4096:(g + 1) * 4096][keep[g * 4096:(g + 1) * 4096]][:k_cap]
        assert np.array_equal(got[g * k_cap:g * k_cap + kept.size], kept)
