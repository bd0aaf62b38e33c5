"""Seeded random shapes against the oracle: prune+pack bit-exact, dW within tolerance.

The fixed shape lists of test_gpu_parity.py follow the paper's networks; this sweep draws unusual combinations
(unpadded and strided filters, odd sizes, few channels, groups that do or do not match the hint) so that every
staging variant of the weight-gradient kernels and every selection path is exercised.  Each case prints its
parameters before it touches the GPU."""
import random

import numpy as np
import pytest
import torch

import oracle
import paper_2503_20354_amd as surgeon
import surgeon_workloads as wl
from parity_bars import assert_dw_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def pack_and_check(A, g, r):
    p = surgeon.prune_pack(A.to(DEV), g, r, want_idx=True)
    torch.cuda.synchronize()
    o_vals, o_mask, o_idx, o_k = oracle.prune_pack(wl.to_numpy_bits(A).reshape(-1), g, r)
    assert p.k_total == o_k
    assert np.array_equal(p.mask.cpu().numpy().view(np.uint64), o_mask), "mask"
    assert np.array_equal(wl.to_numpy_bits(p.vals).view(np.uint8), o_vals.view(np.uint8)), "vals"
    assert np.array_equal(p.idx.cpu().numpy().view(np.uint32), o_idx), "idx"
    return p, o_vals, o_mask


def dw_on_gpu(desc, p, dY, shape):
    dW = torch.empty(shape, device=DEV)
    ws = torch.empty(max(16, surgeon.surgeon_dw_ws_bytes(desc)), dtype=torch.uint8, device=DEV)
    surgeon.surgeon_dw_from_packed(desc, p.vals, p.mask, dY.to(DEV), dW, ws)
    torch.cuda.synchronize()
    return dW.cpu().numpy()


@pytest.mark.parametrize("seed", [101, 102, 103, 104])
def test_random_conv_shapes(seed):
    rng = random.Random(seed)
    done = 0
    while done < 14:
        dtype = rng.choice(["f32", "bf16"])
        dt = surgeon.F32 if dtype == "f32" else surgeon.BF16
        r = rng.choice([0.0, 0.3, 0.5, 0.77, 0.9, 0.97])
        k = rng.choice([1, 1, 3, 3, 3, 5, 7])
        st = rng.choice([1, 1, 1, 2, 2, 3])
        pad = rng.choice([k // 2, k // 2, 0])
        Nb = rng.randint(1, 3)
        Ci = rng.choice([1, 3, 5, 16, 31, 33, 64, 70, 128])
        Co = rng.choice([1, 7, 16, 64, 65, 160, 170])
        H = rng.choice([5, 7, 8, 9, 14, 16, 17, 28, 32, 33, 40, 56])
        W = rng.choice([5, 7, 8, 9, 14, 16, 17, 24, 28, 32, 33, 40, 56, 100])
        if H + 2 * pad < k or W + 2 * pad < k:
            continue
        OH, OW = (H + 2 * pad - k) // st + 1, (W + 2 * pad - k) // st + 1
        if Nb * Co * Ci * k * k * OH * OW > 4e8:
            continue
        n = Nb * Ci * H * W
        g = rng.choice([64, 512, 4096, n, 5000, 100])
        hint = rng.random() < 0.6
        print("conv Nb=%d Ci=%d H=%d W=%d Co=%d k=%d stride=%d pad=%d %s r=%g g=%d hint=%d" %
              (Nb, Ci, H, W, Co, k, st, pad, dtype, r, g, hint), flush=True)
        A = wl.draw((Nb, Ci, H, W), rng.choice(["relu", "normal"]), dtype, seed * 1000 + done * 3 + 1)
        dY = wl.draw((Nb, Co, OH, OW), "normal", dtype, seed * 1000 + done * 3 + 2)
        p, o_vals, o_mask = pack_and_check(A, g, r)
        desc = surgeon.conv2d_desc(Nb, Ci, H, W, Co, k, k, st, pad, dt, p.k_total, group_len=g if hint else 0,
                                   r=r if hint else 0.0)
        got = dw_on_gpu(desc, p, dY, (Co, Ci, k, k))
        ref = oracle.dw_conv2d(o_vals, o_mask, wl.to_numpy_bits(dY), Nb, Ci, H, W, Co, k, k, st, pad)
        assert_dw_close(got, ref, dtype)
        done += 1


@pytest.mark.parametrize("seed", [151, 152, 153])
def test_random_shapes_of_the_kept_elements_kernel(seed):
    """fp32 3x3 stride-1 pad-1 layers of width 8 / 16 / 32 with few kept elements (the kernel that sums Eq. 2 over the
    kept elements only): odd channel counts, partial channel tiles, one to many bands and images, every group scope."""
    rng = random.Random(seed)
    for case in range(12):
        W = rng.choice([8, 16, 32])
        H = rng.choice([1, 2, 3, 5]) * (4 if W == 32 else 8)
        Nb = rng.randint(1, 7)
        Ci = rng.choice([1, 3, 31, 32, 33, 64, 64, 100, 128, 160])
        Co = rng.choice([32, 33, 63, 64, 65, 128, 200])
        r = rng.choice([0.8, 0.85, 0.9, 0.9, 0.95, 0.99, 1.0])
        n = Nb * Ci * H * W
        g = rng.choice([64, 4096, 4096, n, 1000, 128])
        hint = rng.random() < 0.5
        print("kept-elements conv Nb=%d Ci=%d H=%d W=%d Co=%d r=%g g=%d hint=%d" % (Nb, Ci, H, W, Co, r, g, hint), flush=True)
        A = wl.draw((Nb, Ci, H, W), rng.choice(["relu", "normal"]), "f32", seed * 1000 + case * 3 + 1)
        dY = wl.draw((Nb, Co, H, W), "normal", "f32", seed * 1000 + case * 3 + 2)
        p, o_vals, o_mask = pack_and_check(A, g, r)
        desc = surgeon.conv2d_desc(Nb, Ci, H, W, Co, 3, 3, 1, 1, surgeon.F32, p.k_total, group_len=g if hint else 0,
                                   r=r if hint else 0.0)
        if p.k_total * 100 <= 17 * n:
            assert surgeon.surgeon_dw_kernel_class(desc) == "dw_sparse"
        got = dw_on_gpu(desc, p, dY, (Co, Ci, 3, 3))
        ref = oracle.dw_conv2d(o_vals, o_mask, wl.to_numpy_bits(dY), Nb, Ci, H, W, Co, 3, 3, 1, 1)
        assert_dw_close(got, ref, "f32")


@pytest.mark.parametrize("seed", [201, 202])
def test_random_linear_shapes(seed):
    rng = random.Random(seed)
    for case in range(12):
        dtype = rng.choice(["f32", "bf16"])
        dt = surgeon.F32 if dtype == "f32" else surgeon.BF16
        r = rng.choice([0.0, 0.5, 0.9, 0.97, 1.0])
        M = rng.choice([1, 7, 64, 100, 333, 1000])
        K = rng.choice([8, 64, 70, 128, 320, 512, 768])
        N = rng.choice([8, 19, 64, 72, 256, 520])
        g = rng.choice([K, K, 64, M * K, 1000])
        hint = rng.random() < 0.6
        print("linear M=%d K=%d N=%d %s r=%g g=%d hint=%d" % (M, K, N, dtype, r, g, hint), flush=True)
        A = wl.draw((M, K), "normal", dtype, seed * 1000 + case * 3 + 1)
        dY = wl.draw((M, N), "normal", dtype, seed * 1000 + case * 3 + 2)
        p, o_vals, o_mask = pack_and_check(A, g, r)
        desc = surgeon.linear_desc(M, K, N, dt, p.k_total, group_len=g if hint else 0, r=r if hint else 0.0)
        got = dw_on_gpu(desc, p, dY, (N, K))
        ref = oracle.dw_linear(o_vals, o_mask, wl.to_numpy_bits(dY), M, K, N)
        assert_dw_close(got, ref, dtype)


@pytest.mark.parametrize("seed", [301])
def test_random_selection_sizes(seed):
    rng = random.Random(seed)
    for case in range(16):
        dtype = rng.choice(["f32", "bf16"])
        r = rng.choice([0.0, 0.3, 0.5, 0.9, 0.97, 1.0])
        n = rng.choice([1, 63, 4097, 20000, 70001, 300000, 1000000])
        g = rng.choice([n, 4097, 5000, 8192, 20000, 64, 4096, 1000, 65536])
        dist = rng.choice(["relu", "normal", "relu"])
        print("select n=%d g=%d %s %s r=%g" % (n, g, dist, dtype, r), flush=True)
        pack_and_check(wl.draw((n,), dist, dtype, seed * 1000 + case), g, r)
