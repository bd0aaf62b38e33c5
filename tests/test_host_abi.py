"""CPU-only checks of the library's host side: it loads, exports every declared symbol, and its host-only
entry points (size rules, Eq. 5-7, argument errors) agree with the oracle.  No kernel is launched."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2503_20354_amd as surgeon

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "surgeon.h")).read()
    declared = set(re.findall(r"\b(surgeon_[a-z_]+)\s*\(", header))
    assert {"surgeon_layer_ratios", "surgeon_prune_pack", "surgeon_dw_from_packed", "surgeon_grad_importance"} <= declared
    lib = ctypes.CDLL(surgeon.library_path())
    for name in sorted(declared):
        assert hasattr(lib, name), name


def test_keep_count_matches_table_and_oracle():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "keep_count_cases.txt")) if l.strip() and l[0] != "#"]
    for r, length, k in rows:
        assert surgeon.surgeon_keep_count(int(length), float(r)) == int(k)
    rng = np.random.default_rng(0)
    for _ in range(2000):
        length = int(rng.integers(0, 10**7))
        r = float(np.float32(rng.random()))
        assert surgeon.surgeon_keep_count(length, r) == oracle.keep_count(length, r)
    assert surgeon.surgeon_keep_count(10, 1.5) == -1
    assert surgeon.surgeon_keep_count(-3, 0.5) == -1
    assert surgeon.surgeon_keep_count(10, float("nan")) == -1


def test_packed_sizes():
    k, vb, mb, wb = surgeon.surgeon_packed_sizes(32768, 512, 0.5, surgeon.F32)
    assert (k, vb, mb, wb) == (16384, 65536, 4096, 0)
    k, vb, mb, _ = surgeon.surgeon_packed_sizes(1000, 300, 0.9, surgeon.BF16)
    assert k == oracle.total_kept(1000, 300, 0.9) and vb == 2 * k and mb == 8 * 16
    assert surgeon.surgeon_packed_sizes(0, 64, 0.5, surgeon.F32)[:3] == (0, 0, 0)
    # whole-tensor scope needs a workspace, the in-register path does not
    assert surgeon.surgeon_packed_sizes(10**6, 10**6, 0.5, surgeon.F32)[3] > 0
    for bad in [(-1, 64, 0.5, 0), (10, 0, 0.5, 0), (10, 4, 1.5, 0), (10, 4, 0.5, 7), (10, 4, float("nan"), 0)]:
        with pytest.raises(surgeon.SurgeonError) as e:
            surgeon.surgeon_packed_sizes(*bad)
        assert e.value.status == 1
    assert "packed_sizes" in surgeon.surgeon_last_error()


def test_layer_ratios_against_oracle_and_examples():
    for line in open(os.path.join(GOLDEN, "layer_ratio_examples.txt")):
        if not line.strip() or line.startswith("#"):
            continue
        m, G, p = (part.split() for part in line.split("|"))
        got = surgeon.surgeon_layer_ratios([float(x) for x in G], [int(x) for x in m])
        assert np.allclose(got.numpy(), np.array(p, dtype=np.float64), atol=1e-7)
    rng = np.random.default_rng(1)
    for _ in range(50):
        l = int(rng.integers(1, 300))
        m = rng.integers(1, 2**40, l).astype(np.uint64)
        G = (rng.random(l) * 10).astype(np.float32)
        lo, hi = sorted(np.float32(rng.random(2)).tolist())
        got = surgeon.surgeon_layer_ratios(G, m, lo, hi).numpy()
        assert np.allclose(got, oracle.layer_ratios(G, m, lo, hi), atol=1e-6)
        assert (got >= np.float32(lo) - 1e-7).all() and (got <= np.float32(hi) + 1e-7).all()


def test_layer_ratios_errors():
    for args in [([1.0, -1.0], [1, 1]), ([1.0, 1.0], [1, 0]), ([1.0, float("inf")], [1, 1]), ([], [])]:
        with pytest.raises(surgeon.SurgeonError):
            surgeon.surgeon_layer_ratios(*args)
    with pytest.raises(surgeon.SurgeonError):
        surgeon.surgeon_layer_ratios([1.0], [1], 0.9, 0.3)


def test_dw_kernel_class_and_one_workspace_for_all_ratios():
    """The weight-gradient kernel is chosen from the shape and the kept count; the workspace query covers both."""
    n = 8 * 160 * 32 * 32

    def conv(k_total, dt=surgeon.F32, W=32, stride=1, ksz=3, pad=1):
        return surgeon.conv2d_desc(8, 160, 32, W, 160, ksz, ksz, stride, pad, dt, k_total)

    assert surgeon.surgeon_dw_kernel_class(conv(n // 10)) == "dw_sparse"
    assert surgeon.surgeon_dw_kernel_class(conv(n * 17 // 100)) == "dw_sparse"
    assert surgeon.surgeon_dw_kernel_class(conv(n * 17 // 100 + 1)) == "dw"
    assert surgeon.surgeon_dw_kernel_class(conv(n // 2)) == "dw"
    assert surgeon.surgeon_dw_kernel_class(conv(n // 20, dt=surgeon.BF16)) == "dw"
    assert surgeon.surgeon_dw_kernel_class(conv(n // 20, stride=2)) == "dw"
    assert surgeon.surgeon_dw_kernel_class(conv(n // 20, ksz=1, pad=0)) == "dw"
    assert surgeon.surgeon_dw_kernel_class(surgeon.conv2d_desc(8, 160, 32, 24, 160, 3, 3, 1, 1, surgeon.F32, 1000)) == "dw"
    assert surgeon.surgeon_dw_kernel_class(surgeon.linear_desc(64, 512, 256, surgeon.F32, 100)) == "dw"
    # input channels that fill 64-channel workgroups: the kernel that skips dropped elements pays up to 22 % kept
    n2 = 8 * 320 * 16 * 16
    wide = lambda k: surgeon.conv2d_desc(8, 320, 16, 16, 320, 3, 3, 1, 1, surgeon.F32, k)
    assert surgeon.surgeon_dw_kernel_class(wide(n2 * 22 // 100)) == "dw_sparse"
    assert surgeon.surgeon_dw_kernel_class(wide(n2 * 22 // 100 + 1)) == "dw"
    sizes = {surgeon.surgeon_dw_ws_bytes(conv(k)) for k in (0, n // 10, n // 2, n)}
    assert len(sizes) == 1  # sized once, valid for every prune ratio


def test_dw_workspace_and_shape_errors():
    d = surgeon.conv2d_desc(200, 160, 32, 32, 160, 3, 3, 1, 1, surgeon.F32, 1000)
    assert surgeon.surgeon_dw_ws_bytes(d) > 0
    d = surgeon.linear_desc(64, 512, 256, surgeon.F32, 16384)
    assert surgeon.surgeon_dw_ws_bytes(d) >= 4 * (32768 // 64)
    with pytest.raises(surgeon.SurgeonError) as e:
        surgeon.surgeon_dw_ws_bytes(surgeon.conv2d_desc(1, 1, 8, 8, 1, 3, 4, 1, 1, surgeon.F32, 0))
    assert e.value.status == 3  # filter width 4 is not implemented
    with pytest.raises(surgeon.SurgeonError) as e:
        surgeon.surgeon_dw_ws_bytes(surgeon.linear_desc(4, 0, 4, surgeon.F32, 0))
    assert e.value.status == 1
    with pytest.raises(surgeon.SurgeonError):
        surgeon.surgeon_dw_ws_bytes(surgeon.linear_desc(4, 4, 4, surgeon.F32, 17))  # k_total > n


def test_undersized_workspace_is_rejected_before_any_launch():
    """SURGEON_ESIZE comes from the host checks: with a workspace one byte short nothing is launched, so made-up
    (aligned, never dereferenced) pointers are enough and the test needs no GPU."""
    lib = surgeon.load_library()
    fake = lambda k: ctypes.c_void_p(0x10000 * k)
    # weight gradient: conv layer with a split contraction
    d = surgeon.conv2d_desc(200, 160, 32, 32, 160, 3, 3, 1, 1, surgeon.F32, 200 * 160 * 32 * 32 // 2)
    need = surgeon.surgeon_dw_ws_bytes(d)
    assert need > 16
    rc = lib.surgeon_dw_from_packed(ctypes.byref(d), fake(1), fake(2), fake(3), fake(4), fake(5), need - 1, None)
    assert rc == 2 and "workspace" in surgeon.surgeon_last_error()
    rc = lib.surgeon_dw_from_packed(ctypes.byref(d), fake(1), fake(2), fake(3), fake(4), None, 0, None)
    assert rc == 2
    # selection over the whole tensor needs a workspace; groups of at most 4096 elements need none
    n = 1 << 20
    need = surgeon.surgeon_packed_sizes(n, n, 0.5, surgeon.F32)[3]
    assert need > 0
    rc = lib.surgeon_prune_pack(fake(1), n, n, 0.5, surgeon.F32, fake(2), fake(3), None, fake(4), need - 1, None)
    assert rc == 2 and "workspace" in surgeon.surgeon_last_error()
    rc = lib.surgeon_prune_pack(fake(1), n, n, 0.5, surgeon.F32, fake(2), fake(3), None, None, 0, None)
    assert rc == 2
    # Gradient Importance
    need = surgeon.surgeon_grad_importance_ws_bytes(5_000_000)
    if need > 0:
        rc = lib.surgeon_grad_importance(fake(1), 5_000_000, fake(2), fake(3), need - 1, None)
        assert rc == 2
