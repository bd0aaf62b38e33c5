"""GPU parity of the rest of Alg. 1's backward step and of the other layer types, against the CPU oracle:
Gradient Importance folded into the weight-gradient call (Eq. 4 inside Alg. 1 line 12), the activation gradient
dA = dY . W (Eq. 2, first line), the gradient step (Alg. 1 line 14), scale / shift gradients of normalisation layers
(Section 5, the variant that adapts BN layers only) and grouped / depthwise convolution weight gradients.
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


def bits(t):
    return wl.to_numpy_bits(t)


def f64(a):
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def sdt(dtype):
    return surgeon.F32 if dtype == "f32" else surgeon.BF16


def assert_out_close(got_bits, ref_bits, dtype, what=""):
    """Outputs stored in the layer's dtype.  fp32: the dW bars.  bf16: the stated 2e-2 norm bar, a tight one, and per
    entry at most one bf16 step (the oracle rounds the exact sum, the kernel rounds an fp32 sum: they can land on
    neighbouring values, never further apart)."""
    got, ref = f64(got_bits).ravel(), f64(ref_bits).ravel()
    if dtype == "f32":
        assert_dw_close(got, ref, "f32", what)
        return
    e = rel_l2(got, ref)
    assert e <= TOL["bf16"], (what, e)
    assert e <= 2e-3, (what, e)
    step = np.maximum(np.abs(ref), 1e-30) * 2.0 ** -7  # one bf16 step is at most 2^-7 of the value
    worst = np.abs(got - ref) - step
    floor = 1e-5 * float(np.abs(ref).max())            # sums that cancel to ~0: an absolute floor from the fp32 accumulation
    assert (worst <= floor).all(), (what, float(worst.max()), floor)


# ------------------------------------------------------------------------------------------------
# Eq. 4 inside the weight-gradient call
# ------------------------------------------------------------------------------------------------
def _dw_gi(desc, p, dY):
    shape = (desc.N, desc.K) if desc.kind == 0 else (desc.Co, desc.Ci // max(desc.groups, 1), desc.kh, desc.kw)
    desc.group_len, desc.r = p.group_len, p.r
    plain = torch.empty(shape, device=DEV)
    fused = torch.empty(shape, device=DEV)
    G = torch.full((1,), -1.0, device=DEV)
    ws = torch.empty(surgeon.surgeon_dw_gi_ws_bytes(desc), dtype=torch.uint8, device=DEV)
    surgeon.surgeon_dw_from_packed(desc, p.vals, p.mask, dY, plain, ws)
    surgeon.surgeon_dw_from_packed_gi(desc, p.vals, p.mask, dY, fused, G, ws)
    G2 = torch.full((1,), -2.0, device=DEV)
    again = torch.empty(shape, device=DEV)
    surgeon.surgeon_dw_from_packed_gi(desc, p.vals, p.mask, dY, again, G2, ws)
    torch.cuda.synchronize()
    assert torch.equal(plain, fused) and torch.equal(fused, again)  # same bits with and without, and call after call
    assert G.item() == G2.item()
    return fused.cpu().numpy(), G.item()


GI_CONVS = [
    # Nb, Ci, H, W, Co, k, stride, dtype, r   (the first ones split the contraction, the small ones do not)
    (16, 160, 32, 32, 160, 3, 1, "f32", 0.5), (16, 160, 32, 32, 160, 3, 1, "f32", 0.9), (8, 64, 56, 56, 256, 1, 1, "bf16", 0.8),
    (2, 3, 32, 32, 16, 3, 1, "f32", 0.3), (4, 128, 28, 28, 128, 3, 2, "bf16", 0.7), (1, 8, 8, 8, 8, 3, 1, "f32", 0.5),
    (3, 40, 16, 16, 64, 3, 1, "f32", 1.0),
]


@pytest.mark.parametrize("case", GI_CONVS)
def test_gradient_importance_inside_the_conv_weight_gradient(case):
    Nb, Ci, H, W, Co, k, st, dtype, r = case
    print("dw_gi conv", case, flush=True)
    pad = k // 2
    OH, OW = (H + 2 * pad - k) // st + 1, (W + 2 * pad - k) // st + 1
    A = wl.draw((Nb, Ci, H, W), "relu", dtype, sum(case[:7]) + 1)
    dY = wl.draw((Nb, Co, OH, OW), "normal", dtype, sum(case[:7]) + 2)
    p = surgeon.prune_pack(A.to(DEV), 4096, r)
    desc = surgeon.conv2d_desc(Nb, Ci, H, W, Co, k, k, st, pad, sdt(dtype), p.k_total)
    dW, G = _dw_gi(desc, p, dY.to(DEV))
    o_vals, o_mask, _, _ = oracle.prune_pack(bits(A).reshape(-1), 4096, r)
    ref = oracle.dw_conv2d(o_vals, o_mask, bits(dY), Nb, Ci, H, W, Co, k, k, st, pad)
    assert_dw_close(dW, ref, dtype, case)
    o_G = oracle.grad_importance(ref)
    assert abs(G - o_G) <= 1e-5 * max(o_G, 1e-30)
    if r == 1.0:
        assert G == 0.0 and not dW.any()


@pytest.mark.parametrize("M,K,N,dtype,r", [(4096, 768, 2304, "bf16", 0.9), (2000, 320, 1280, "bf16", 0.6),
                                            (64, 512, 256, "f32", 0.5), (3000, 64, 64, "bf16", 0.7), (500, 96, 40, "f32", 0.0)])
def test_gradient_importance_inside_the_linear_weight_gradient(M, K, N, dtype, r):
    print("dw_gi linear", (M, K, N, dtype, r), flush=True)
    A = wl.draw((M, K), "normal", dtype, M + K + 1)
    dY = wl.draw((M, N), "normal", dtype, M + K + 2)
    p = surgeon.prune_pack(A.to(DEV), K, r)
    dW, G = _dw_gi(surgeon.linear_desc(M, K, N, sdt(dtype), p.k_total), p, dY.to(DEV))
    o_vals, o_mask, _, _ = oracle.prune_pack(bits(A).reshape(-1), K, r)
    ref = oracle.dw_linear(o_vals, o_mask, bits(dY), M, K, N)
    assert_dw_close(dW, ref, dtype, (M, K, N))
    o_G = oracle.grad_importance(ref)
    assert abs(G - o_G) <= 1e-5 * o_G


# ------------------------------------------------------------------------------------------------
# activation gradient (Eq. 2, first line)
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,K,N", [(64, 512, 256), (100, 70, 50), (300, 129, 257), (1, 64, 64), (517, 320, 1280),
                                   (1000, 768, 19), (129, 8, 8),
                                   # bf16 with N % 8 == 0: dY read in place on the bf16 matrix cores; K that 8 does
                                   # not divide (element-wise loads of W), rows and columns that leave tiles part empty
                                   (130, 100, 72), (1000, 768, 96), (200, 65, 64), (257, 136, 200), (64, 64, 64)])
def test_da_linear(dtype, M, K, N):
    print("da linear", (M, K, N), dtype, flush=True)
    dY = wl.draw((M, N), "normal", dtype, M + N + 5)
    W = wl.draw((N, K), "normal", dtype, N + K + 6) * 0.1
    W = W.to(dY.dtype)
    dA = torch.empty((M, K), dtype=dY.dtype, device=DEV)
    surgeon.surgeon_da(surgeon.linear_desc(M, K, N, sdt(dtype), 0), dY.to(DEV), W.to(DEV), dA)
    torch.cuda.synchronize()
    ref = oracle.da_linear(bits(dY), bits(W), M, K, N)
    assert_out_close(bits(dA), ref, dtype, (M, K, N))


@pytest.mark.parametrize("M,K,N", [(256, 64, 64), (1000, 768, 96), (520, 320, 1280), (4096, 128, 512), (264, 72, 200),
                                   (12608, 768, 768), (300, 129, 257), (100, 64, 64)])
def test_da_linear_with_workspace(M, K, N):
    """bf16 linear layers through the workspace entry: shapes that take the bf16 matrix cores (several tiles, ragged
    tiles, a split contraction) and shapes that fall back to the workspace-less route, against the oracle and against
    surgeon_da to one bf16 rounding."""
    print("da_ws linear", (M, K, N), flush=True)
    dY = wl.draw((M, N), "normal", "bf16", M + N + 15)
    W = (wl.draw((N, K), "normal", "bf16", N + K + 16) * 0.1).to(dY.dtype)
    desc = surgeon.linear_desc(M, K, N, sdt("bf16"), 0)
    nb = surgeon.surgeon_da_ws_bytes(desc)
    fast = M >= 256 and M % 8 == 0 and K % 8 == 0 and K >= 64 and N >= 64
    assert (nb > 0) == fast
    ws = torch.empty(max(nb, 16), dtype=torch.uint8, device=DEV)
    dA = torch.empty((M, K), dtype=dY.dtype, device=DEV)
    dA2 = torch.empty_like(dA)
    dYd, Wd = dY.to(DEV), W.to(DEV)
    surgeon.surgeon_da_ws(desc, dYd, Wd, dA, ws)
    surgeon.surgeon_da(desc, dYd, Wd, dA2)
    torch.cuda.synchronize()
    if M <= 4096:
        ref = oracle.da_linear(bits(dY), bits(W), M, K, N)
        assert_out_close(bits(dA), ref, "bf16", (M, K, N))
    # the two routes differ in fp32 summation order only: at most one bf16 rounding step apart (sums that cancel to
    # about zero: the absolute floor of the fp32 accumulation, as in assert_out_close)
    assert_out_close(bits(dA), bits(dA2), "bf16", ("two routes", M, K, N))
    if fast:
        with pytest.raises(surgeon.SurgeonError):
            surgeon.surgeon_da_ws(desc, dYd, Wd, dA, ws[: nb - 256])


DA_CONVS = [
    # Nb, Ci, H, W, Co, k, stride, pad
    (2, 16, 32, 32, 160, 3, 1, 1), (2, 160, 16, 16, 160, 3, 1, 1), (2, 160, 32, 32, 320, 3, 2, 1), (2, 16, 32, 32, 160, 1, 1, 0),
    (2, 160, 32, 32, 320, 1, 2, 0), (2, 3, 32, 32, 16, 3, 1, 1), (1, 3, 64, 64, 64, 7, 2, 3), (2, 64, 14, 14, 256, 1, 1, 0),
    (2, 5, 9, 9, 7, 5, 1, 2), (3, 6, 12, 12, 20, 3, 1, 0), (2, 40, 13, 13, 24, 3, 1, 1), (2, 8, 20, 20, 24, 5, 2, 1),
    (1, 64, 14, 14, 65, 3, 3, 1), (2, 130, 7, 7, 512, 3, 1, 1),
    # 3x3 stride-1 pad-1 layers on maps the band kernel takes: every channel tile (64, 128, 160), 64 and 128 positions
    # per band, channel counts that neither the tile nor the eight-channel step divides, maps 8 to 128 wide
    (3, 130, 8, 8, 13, 3, 1, 1), (2, 24, 16, 8, 20, 3, 1, 1), (1, 8, 4, 64, 9, 3, 1, 1), (1, 5, 3, 128, 6, 3, 1, 1),
    (2, 160, 8, 8, 24, 3, 1, 1), (1, 12, 4, 16, 8, 3, 1, 1), (2, 320, 16, 16, 40, 3, 1, 1), (4, 24, 4, 16, 16, 3, 1, 1),
    # ... and maps that leave part of a tile empty: a short last band, a last tile with fewer images, tiny and wide maps
    (3, 20, 14, 14, 24, 3, 1, 1), (5, 8, 7, 7, 8, 3, 1, 1), (1, 6, 56, 56, 10, 3, 1, 1), (9, 6, 4, 4, 8, 3, 1, 1),
    (1, 5, 5, 100, 4, 3, 1, 1), (2, 5, 3, 3, 4, 3, 1, 1), (1, 7, 1, 1, 5, 3, 1, 1), (2, 7, 40, 2, 9, 3, 1, 1),
    # 1x1 layers, stride 1 and 2 (bf16: the matrix-core route): channel counts and maps that 8 does not divide, odd maps
    # under stride 2 (the last row and column of dA have no partner), more channels than one tile
    (3, 20, 7, 7, 33, 1, 1, 0), (2, 24, 7, 7, 16, 1, 2, 0), (1, 130, 9, 5, 70, 1, 2, 0), (2, 264, 14, 14, 100, 1, 1, 0),
    (2, 8, 28, 28, 300, 1, 2, 0),
    # at most four input channels (the per-pixel kernel): strides, pads and filter sizes
    (2, 4, 9, 9, 6, 3, 2, 0), (3, 1, 5, 7, 3, 5, 1, 2), (2, 2, 6, 6, 5, 1, 1, 0), (1, 3, 37, 41, 70, 7, 2, 3),
    # 3x3 stride-2 pad-1 layers (the cell kernel): even and odd maps, bands that do not fill a tile, 64- and 80-channel
    # tiles with channels left over, the widest map it takes and one past it
    (2, 24, 14, 14, 20, 3, 2, 1), (3, 70, 9, 7, 12, 3, 2, 1), (1, 8, 6, 128, 5, 3, 2, 1), (1, 8, 6, 130, 5, 3, 2, 1),
    (2, 96, 32, 16, 40, 3, 2, 1), (2, 80, 16, 16, 33, 3, 2, 1), (1, 5, 1, 1, 4, 3, 2, 1),
    # strided 1x1 layers outside the bf16 stride-2 route: stride 3, maps the stride does not divide
    (2, 9, 10, 7, 12, 1, 3, 0), (1, 140, 15, 15, 30, 1, 2, 0),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", DA_CONVS)
def test_da_conv(dtype, case):
    Nb, Ci, H, W, Co, k, st, pad = case
    print("da conv", case, dtype, flush=True)
    OH, OW = (H + 2 * pad - k) // st + 1, (W + 2 * pad - k) // st + 1
    dY = wl.draw((Nb, Co, OH, OW), "normal", dtype, sum(case) + 5)
    Wt = (wl.draw((Co, Ci, k, k), "normal", dtype, sum(case) + 6) * 0.1).to(dY.dtype)
    dA = torch.empty((Nb, Ci, H, W), dtype=dY.dtype, device=DEV)
    surgeon.surgeon_da(surgeon.conv2d_desc(Nb, Ci, H, W, Co, k, k, st, pad, sdt(dtype), 0), dY.to(DEV), Wt.to(DEV), dA)
    torch.cuda.synchronize()
    ref = oracle.da_conv2d(bits(dY), bits(Wt), Nb, Ci, H, W, Co, k, k, st, pad)
    assert_out_close(bits(dA), ref, dtype, case)


@pytest.mark.parametrize("seed", [401, 402, 403])
def test_da_random_conv_shapes(seed):
    """Seeded random layers over every route of the activation gradient (3x3 band and stride-2 cell kernels with
    partly filled tiles, bf16 1x1 on the bf16 matrix cores with aligned and unaligned maps, few input channels,
    strided 1x1 spread, the gathering kernel).  Each case prints its parameters before it touches the GPU."""
    import random
    rng = random.Random(seed)
    done = 0
    while done < 16:
        dtype = rng.choice(["f32", "bf16"])
        k, st, pad = rng.choice([(3, 1, 1), (3, 1, 1), (3, 2, 1), (3, 2, 1), (1, 1, 0), (1, 2, 0), (1, 3, 0), (3, 1, 0), (5, 2, 2)])
        Nb = rng.randint(1, 5)
        Ci = rng.choice([1, 3, 4, 5, 16, 31, 64, 80, 96, 130, 160, 200])
        Co = rng.choice([1, 7, 8, 9, 24, 64, 100])
        H = rng.choice([1, 2, 4, 7, 8, 9, 14, 16, 17, 28, 32, 33])
        W = rng.choice([1, 2, 4, 7, 8, 9, 14, 16, 17, 28, 32, 33, 64, 100, 128, 130])
        if H + 2 * pad < k or W + 2 * pad < k:
            continue
        OH, OW = (H + 2 * pad - k) // st + 1, (W + 2 * pad - k) // st + 1
        if Nb * Co * Ci * k * k * OH * OW > 2e8:
            continue
        case = (Nb, Ci, H, W, Co, k, st, pad)
        print("da random conv", case, dtype, flush=True)
        dY = wl.draw((Nb, Co, OH, OW), "normal", dtype, seed * 1000 + 2 * done)
        Wt = (wl.draw((Co, Ci, k, k), "normal", dtype, seed * 1000 + 2 * done + 1) * 0.1).to(dY.dtype)
        dA = torch.full((Nb, Ci, H, W), float("nan"), dtype=dY.dtype, device=DEV)  # every element must be overwritten
        surgeon.surgeon_da(surgeon.conv2d_desc(Nb, Ci, H, W, Co, k, k, st, pad, sdt(dtype), 0), dY.to(DEV), Wt.to(DEV), dA)
        torch.cuda.synchronize()
        ref = oracle.da_conv2d(bits(dY), bits(Wt), Nb, Ci, H, W, Co, k, k, st, pad)
        assert_out_close(bits(dA), ref, dtype, case)
        done += 1


DA_GROUPED = [
    # Nb, Ci, H, W, Co, k, stride, pad, groups
    (2, 64, 16, 16, 64, 3, 1, 1, 8), (2, 32, 9, 9, 64, 3, 2, 1, 4), (3, 40, 12, 10, 40, 3, 1, 1, 40), (1, 12, 7, 7, 24, 5, 2, 2, 3),
    (2, 8, 8, 8, 8, 1, 1, 0, 2), (1, 130, 33, 17, 130, 3, 1, 1, 130), (2, 6, 40, 40, 12, 7, 1, 3, 6),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", DA_GROUPED)
def test_da_grouped_conv(dtype, case):
    """Activation gradient of grouped and depthwise layers against the oracle (outputs pre-filled with NaN)."""
    Nb, Ci, H, W, Co, k, st, pad, groups = case
    print("da grouped conv", case, dtype, flush=True)
    OH, OW = (H + 2 * pad - k) // st + 1, (W + 2 * pad - k) // st + 1
    dY = wl.draw((Nb, Co, OH, OW), "normal", dtype, sum(case) + 15)
    Wt = (wl.draw((Co, Ci // groups, k, k), "normal", dtype, sum(case) + 16) * 0.1).to(dY.dtype)
    dA = torch.full((Nb, Ci, H, W), float("nan"), dtype=dY.dtype, device=DEV)
    desc = surgeon.conv2d_desc(Nb, Ci, H, W, Co, k, k, st, pad, sdt(dtype), 0, groups=groups)
    surgeon.surgeon_da(desc, dY.to(DEV), Wt.to(DEV), dA)
    torch.cuda.synchronize()
    ref = oracle.da_conv2d_grouped(bits(dY), bits(Wt), Nb, Ci, H, W, Co, k, k, st, pad, groups)
    assert_out_close(bits(dA), ref, dtype, case)
    with pytest.raises(surgeon.SurgeonError):  # groups that do not divide the channels
        surgeon.surgeon_da(surgeon.conv2d_desc(Nb, Ci, H, W, Co, k, k, st, pad, sdt(dtype), 0, groups=groups + 1 if Ci % (groups + 1) else 7 * Ci),
                           dY.to(DEV), Wt.to(DEV), dA)


@pytest.mark.parametrize("cfg,name", [(1, "s2b1.conv1"), (1, "s3b2.conv2"), (2, "s2b1.conv2"), (2, "s3b2.conv3"),
                                      (3, "blk0.qkv"), (3, "blk11.fc2"), (4, "st1b1.fc1"), (4, "dec.cls")])
def test_da_full_size_sampled(cfg, name):
    """One layer of each kind at the benchmark's full size: sampled entries from the definition."""
    layers = wl.config_layers(cfg)
    li = [l.name for l in layers].index(name)
    L = layers[li]
    print("da full size", cfg, name, flush=True)
    _, dY = wl.layer_tensors(cfg, li, L)
    Wt = (wl.draw(L.dw_shape, "normal", L.dtype, 777 + li) * 0.05).to(dY.dtype)
    dA = torch.empty(L.a_shape, dtype=dY.dtype, device=DEV)
    where = np.random.default_rng(li).integers(0, L.n, 2048)
    if L.kind == "linear":
        surgeon.surgeon_da(surgeon.linear_desc(L.M, L.K, L.N, sdt(L.dtype), 0), dY.to(DEV), Wt.to(DEV), dA)
        ref = oracle.da_linear_at(bits(dY), bits(Wt), L.M, L.K, L.N, where)
    else:
        surgeon.surgeon_da(surgeon.conv2d_desc(L.Nb, L.Ci, L.H, L.W, L.Co, L.kh, L.kw, L.stride, L.pad, sdt(L.dtype), 0),
                           dY.to(DEV), Wt.to(DEV), dA)
        ref = oracle.da_conv2d_at(bits(dY), bits(Wt), L.Nb, L.Ci, L.H, L.W, L.Co, L.kh, L.kw, L.stride, L.pad, where)
    torch.cuda.synchronize()
    assert_out_close(bits(dA).reshape(-1)[where], ref, L.dtype, (cfg, name))


# ------------------------------------------------------------------------------------------------
# gradient step (Alg. 1 line 14)
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n", [1, 255, 4097, 1_000_003])
def test_weight_update(dtype, n):
    W = wl.draw((n,), "normal", dtype, n + 1)
    dW = wl.draw((n,), "normal", "f32", n + 2)
    lr = 0.0123
    Wd = W.to(DEV).clone()
    surgeon.surgeon_weight_update(Wd, dW.to(DEV), lr)
    torch.cuda.synchronize()
    ref = oracle.weight_update(bits(W), dW.numpy(), lr)
    got, ref = f64(bits(Wd)), f64(ref)
    # one fused multiply-add in fp32 against the oracle's double arithmetic: at most one unit in the last place apart
    ulp = np.abs(ref) * (2.0 ** -23 if dtype == "f32" else 2.0 ** -7) + 1e-30
    assert (np.abs(got - ref) <= ulp).all()
    assert rel_l2(got, ref) <= (1e-5 if dtype == "f32" else 2e-3)
    same = W.to(DEV).clone()
    surgeon.surgeon_weight_update(same, torch.zeros(n, device=DEV), lr)  # a zero gradient changes nothing
    assert torch.equal(same.cpu(), W)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n_layers", [1, 5, 70, 150])
def test_weight_update_batched(dtype, n_layers):
    """Many tensors per launch (more than 64 take several): the oracle's step per tensor, and the same bits as one call
    per tensor; sizes around the 4096-element chunk, empty tensors, and pointers that rule out 16-byte accesses."""
    rng = np.random.default_rng(n_layers)
    sizes = [int(x) for x in rng.choice([0, 1, 3, 4095, 4096, 4097, 8192, 12289, 36864, 100003], n_layers)]
    sizes[0] = 100003
    lr = 0.0371
    Ws = [wl.draw((n + 1,), "normal", dtype, 500 + i) for i, n in enumerate(sizes)]
    dWs = [wl.draw((n + 1,), "normal", "f32", 900 + i) for i, n in enumerate(sizes)]
    # every third tensor starts one element into its allocation
    off = [1 if i % 3 == 1 else 0 for i in range(n_layers)]
    W_dev = [w.to(DEV).clone() for w in Ws]
    dW_dev = [g.to(DEV) for g in dWs]
    W_view = [w[o:o + n] for w, o, n in zip(W_dev, off, sizes)]
    dW_view = [g[o:o + n] for g, o, n in zip(dW_dev, off, sizes)]
    single = [w.clone() for w in W_dev]
    surgeon.surgeon_weight_update_batched(W_view, dW_view, lr)
    for w, o, n, g in zip(single, off, sizes, dW_view):
        surgeon.surgeon_weight_update(w[o:o + n], g, lr)
    torch.cuda.synchronize()
    for i, n in enumerate(sizes):
        assert torch.equal(W_dev[i].cpu().view(torch.uint8), single[i].cpu().view(torch.uint8)), i
        o = off[i]
        got_all = W_dev[i].cpu()
        # elements outside the view are untouched
        assert torch.equal(got_all[:o], Ws[i][:o]) and torch.equal(got_all[o + n:], Ws[i][o + n:])
        if n == 0:
            continue
        ref = f64(oracle.weight_update(bits(Ws[i][o:o + n]), dWs[i][o:o + n].numpy(), lr))
        got = f64(bits(got_all[o:o + n]))
        ulp = np.abs(ref) * (2.0 ** -23 if dtype == "f32" else 2.0 ** -7) + 1e-30
        assert (np.abs(got - ref) <= ulp).all(), i


# ------------------------------------------------------------------------------------------------
# scale / shift gradients of normalisation layers
# ------------------------------------------------------------------------------------------------
AFFINE_CASES = [
    # outer, C, inner, group_len        batch norm: (Nb, C, H*W); layer norm: (tokens, C, 1)
    (8, 160, 1024, 4096), (5, 64, 64, 4096), (200, 16, 1024, 4096), (3, 7, 49, 1000), (2, 33, 196, 4096),
    (1000, 768, 1, 768), (333, 64, 1, 64), (77, 320, 1, 320), (50, 19, 1, 19), (64, 100, 1, 4096), (1, 1, 1, 1),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", AFFINE_CASES)
def test_affine_grad(dtype, case):
    outer, C, inner, g = case
    for r in (0.0, 0.7, 1.0):
        print("affine_grad", case, dtype, "r=%g" % r, flush=True)
        x = wl.draw((outer, C, inner), "normal", dtype, sum(case) + 1)
        dY = wl.draw((outer, C, inner), "normal", dtype, sum(case) + 2)
        p = surgeon.prune_pack(x.to(DEV), g, r)
        dgamma, dbeta = surgeon.affine_grad(p, dY.to(DEV), outer, C, inner)
        torch.cuda.synchronize()
        o_vals, o_mask, _, o_k = oracle.prune_pack(bits(x).reshape(-1), g, r)
        assert o_k == p.k_total
        rg, rb = oracle.affine_grad(o_vals, o_mask, bits(dY), outer, C, inner)
        # fp32 sums over up to 2e5 terms per channel: compared with the size of what is summed
        scale = max(float(np.sqrt(outer * inner)), 1.0)
        assert np.abs(dgamma.cpu().numpy() - rg).max() <= 1e-5 * scale * max(1.0, float(np.abs(rg).max()) / scale), case
        assert np.abs(dbeta.cpu().numpy() - rb).max() <= 1e-5 * scale * max(1.0, float(np.abs(rb).max()) / scale), case
        if outer * inner >= 64:
            assert rel_l2(dgamma.cpu().numpy(), rg) <= 1e-5 or r == 1.0
            assert rel_l2(dbeta.cpu().numpy(), rb) <= 1e-5
        if r == 1.0:
            assert not dgamma.any().item()


# ------------------------------------------------------------------------------------------------
# grouped and depthwise convolutions
# ------------------------------------------------------------------------------------------------
GROUPED = [
    # Nb, Ci, H, W, Co, k, stride, pad, groups
    (8, 128, 16, 16, 128, 3, 1, 1, 32), (4, 256, 8, 8, 512, 3, 2, 1, 32), (2, 64, 32, 32, 64, 3, 1, 1, 64),
    (2, 320, 16, 32, 320, 3, 1, 1, 320), (3, 12, 9, 9, 24, 5, 2, 2, 4), (2, 6, 11, 11, 6, 7, 1, 3, 6),
    (2, 8, 8, 8, 8, 1, 1, 0, 2), (1, 4, 5, 5, 4, 3, 1, 0, 4),
    # the tiled 3x3 kernel: a last workgroup with fewer groups, more output than input channels per group, bands that
    # do not divide the map, many tiles per split
    (3, 24, 12, 12, 24, 3, 1, 1, 6), (2, 32, 10, 10, 64, 3, 1, 1, 8), (1, 16, 72, 64, 16, 3, 1, 1, 4),
    (40, 64, 8, 8, 64, 3, 1, 1, 8), (3, 100, 12, 12, 100, 3, 1, 1, 100),
    # the depthwise 3x3 kernel: bands of unequal height, maps whose width is no power of two, planes that start inside a
    # mask word, fewer units than wavefronts, many units per split, a wide map with short bands
    (1, 40, 70, 64, 40, 3, 1, 1, 40), (2, 7, 7, 7, 7, 3, 1, 1, 7), (1, 3, 5, 200, 3, 3, 1, 1, 3), (50, 16, 14, 14, 16, 3, 1, 1, 16),
    (1, 2, 1, 1, 2, 3, 1, 1, 2), (2, 1280, 16, 16, 1280, 3, 1, 1, 1280),
]


def test_dw_depthwise_large_layer_without_packing_hint():
    """41.9 M elements and no (group_len, r) in the descriptor: the rank table of a tensor this large comes from the
    three-launch prefix sum (smaller ones fuse the middle launch away), and the depthwise kernel walks 10 bands per
    plane."""
    Nb, C, H, W = 1, 640, 256, 256
    print("dw depthwise large, no hint", (Nb, C, H, W), flush=True)
    A = wl.draw((Nb, C, H, W), "relu", "bf16", 901)
    dY = wl.draw((Nb, C, H, W), "normal", "bf16", 902)
    p = surgeon.prune_pack(A.to(DEV), 4096, 0.9)
    desc = surgeon.conv2d_desc(Nb, C, H, W, C, 3, 3, 1, 1, surgeon.BF16, p.k_total, groups=C)
    dW = torch.empty((C, 1, 3, 3), device=DEV)
    ws = torch.empty(max(16, surgeon.surgeon_dw_ws_bytes(desc)), dtype=torch.uint8, device=DEV)
    surgeon.surgeon_dw_from_packed(desc, p.vals, p.mask, dY.to(DEV), dW, ws)
    torch.cuda.synchronize()
    o_vals, o_mask, _, _ = oracle.prune_pack(bits(A).reshape(-1), 4096, 0.9)
    ref = oracle.dw_conv2d_grouped(o_vals, o_mask, bits(dY), Nb, C, H, W, C, 3, 3, 1, 1, C)
    assert_dw_close(dW.cpu().numpy(), ref, "bf16", "depthwise large")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", GROUPED)
def test_dw_grouped_conv(dtype, case):
    Nb, Ci, H, W, Co, k, st, pad, groups = case
    OH, OW = (H + 2 * pad - k) // st + 1, (W + 2 * pad - k) // st + 1
    for r in (0.0, 0.8, 1.0):
        print("dw grouped", case, dtype, "r=%g" % r, flush=True)
        A = wl.draw((Nb, Ci, H, W), "relu", dtype, sum(case) + 1)
        dY = wl.draw((Nb, Co, OH, OW), "normal", dtype, sum(case) + 2)
        p = surgeon.prune_pack(A.to(DEV), 4096, r)
        desc = surgeon.conv2d_desc(Nb, Ci, H, W, Co, k, k, st, pad, sdt(dtype), p.k_total, groups=groups)
        assert surgeon.surgeon_dw_kernel_class(desc) == "dw_grouped"
        dW, G = _dw_gi(desc, p, dY.to(DEV))
        o_vals, o_mask, _, _ = oracle.prune_pack(bits(A).reshape(-1), 4096, r)
        ref = oracle.dw_conv2d_grouped(o_vals, o_mask, bits(dY), Nb, Ci, H, W, Co, k, k, st, pad, groups)
        assert dW.shape == ref.shape
        assert_dw_close(dW, ref, dtype, case)
        o_G = oracle.grad_importance(ref)
        assert abs(G - o_G) <= 1e-5 * max(o_G, 1e-30)
        # without the packing's (group_len, r) in the descriptor the rank table comes from the general prefix sum
        # instead of the closed form: the same table, so the same bits
        desc.group_len, desc.r = 0, 0.0
        plain = torch.empty(dW.shape, device=DEV)
        ws = torch.empty(max(16, surgeon.surgeon_dw_ws_bytes(desc)), dtype=torch.uint8, device=DEV)
        surgeon.surgeon_dw_from_packed(desc, p.vals, p.mask, dY.to(DEV), plain, ws)
        torch.cuda.synchronize()
        assert np.array_equal(plain.cpu().numpy(), dW), (case, "hint vs no hint")
