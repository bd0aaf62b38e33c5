"""Pins for the oracle's selection and packing (Alg. 1 lines 6-7) -- CPU only.

The oracle sorts; the pins below never sort: they count, for every element, how many elements of its group
beat it, which characterises the unique answer under the order (|a| bit pattern descending, index ascending).
"""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _keys(a):
    if a.dtype == np.float32:
        return a.view(np.uint32) & np.uint32(0x7FFFFFFF)
    return (a & np.uint16(0x7FFF)).astype(np.uint32)


def _bits(mask, n):
    return np.unpackbits(mask.view(np.uint8), bitorder="little")[:n].astype(bool)


def brute_force_keep(a, group_len, r):
    """O(len^2) rank counting: element e is kept iff fewer than k elements of its group beat it."""
    n = a.size
    keys = _keys(a).astype(np.int64)
    keep = np.zeros(n, dtype=bool)
    for start in range(0, n, group_len):
        k_grp = keys[start:start + group_len]
        length = k_grp.size
        k = oracle.keep_count(length, r)
        pos = np.arange(length)
        greater = k_grp[None, :] > k_grp[:, None]
        tie_before = (k_grp[None, :] == k_grp[:, None]) & (pos[None, :] < pos[:, None])
        beats = (greater | tie_before).sum(axis=1)
        keep[start:start + length] = beats < k
    return keep


def _bf16(x):
    """float32 -> bfloat16 bit patterns (round to nearest even), as uint16."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return u.astype(np.uint16)


def test_keep_count_table():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "keep_count_cases.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) >= 15
    for r, length, k in rows:
        assert oracle.keep_count(int(length), float(r)) == int(k), (r, length, k)


def test_keep_count_edges():
    for length in (0, 1, 63, 64, 4096, 10**9):
        assert oracle.keep_count(length, 0.0) == length
        assert oracle.keep_count(length, 1.0) == 0
    assert oracle.keep_count(-1, 0.5) == -1
    assert oracle.keep_count(10, 1.5) == -1
    assert oracle.keep_count(10, float("nan")) == -1
    # monotone: more pruning never keeps more
    ks = [oracle.keep_count(777, r) for r in np.linspace(0, 1, 101)]
    assert all(a >= b for a, b in zip(ks, ks[1:]))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n,g", [(16, 16), (64, 16), (100, 32), (300, 128), (1000, 1000), (257, 64), (4096, 4096)])
def test_selection_matches_rank_counting(dtype, n, g):
    rng = np.random.default_rng(n * 31 + g)
    for r in (0.0, 0.1, 0.5, 0.7, 0.9, 0.95, 1.0):
        x = rng.standard_normal(n).astype(np.float32)
        # force ties: duplicates, +-0, equal magnitudes of opposite sign
        x[rng.integers(0, n, n // 4)] = 0.0
        x[rng.integers(0, n, n // 8)] = -0.0
        j = rng.integers(0, n, n // 6)
        x[j] = -x[(j + 3) % n]
        a = x if dtype == "f32" else _bf16(x)
        vals, mask, idx, k = oracle.prune_pack(a, g, r)
        keep = brute_force_keep(a, g, r)
        assert np.array_equal(_bits(mask, n), keep)
        assert k == keep.sum() == oracle.total_kept(n, g, r)
        # values are the bit-exact kept elements in ascending index; idx is the offset inside the group
        assert np.array_equal(vals.view(np.uint8), a[keep].view(np.uint8))
        assert np.array_equal(idx, (np.nonzero(keep)[0] % g).astype(np.uint32))
        # padding bits of the last word are zero
        assert _bits(mask, mask.size * 64)[n:].sum() == 0


def test_exhaustive_tiny():
    """Every tensor over a 3-letter alphabet with n = 6, every k: the kept set is the one rank counting gives."""
    import itertools
    alphabet = np.array([0.0, -1.0, 1.0, 2.0], dtype=np.float32)
    for combo in itertools.product(range(4), repeat=6):
        a = alphabet[list(combo)]
        for r in (0.0, 0.2, 0.5, 0.8, 1.0):
            _, mask, _, _ = oracle.prune_pack(a, 6, r)
            assert np.array_equal(_bits(mask, 6), brute_force_keep(a, 6, r))


def test_threshold_characterisation_and_nesting():
    rng = np.random.default_rng(7)
    n, g = 8192, 1024
    a = np.maximum(rng.standard_normal(n), 0).astype(np.float32)  # post-ReLU: about half exact zeros
    keys = _keys(a).astype(np.int64)
    prev = None
    for r in (0.0, 0.3, 0.5, 0.6, 0.9, 0.99):
        _, mask, _, _ = oracle.prune_pack(a, g, r)
        keep = _bits(mask, n)
        for s in range(0, n, g):
            kk, kp = keys[s:s + g], keep[s:s + g]
            assert kp.sum() == oracle.keep_count(g, r)
            if kp.any() and (~kp).any():
                assert kk[kp].min() >= kk[~kp].max()
                t = kk[kp].min()
                tied_kept, tied_drop = np.nonzero(kp & (kk == t))[0], np.nonzero(~kp & (kk == t))[0]
                if tied_kept.size and tied_drop.size:
                    assert tied_kept.max() < tied_drop.min()  # lowest index wins a tie
        if prev is not None:
            assert not (keep & ~prev).any()  # larger ratio keeps a subset
        prev = keep


def test_all_equal_and_all_zero_keep_lowest_indices():
    for value in (0.0, -0.0, 3.5):
        a = np.full(100, value, dtype=np.float32)
        vals, mask, idx, k = oracle.prune_pack(a, 100, 0.7)
        assert k == oracle.keep_count(100, 0.7)
        assert np.array_equal(np.nonzero(_bits(mask, 100))[0], np.arange(k))
        assert np.array_equal(vals.view(np.uint32), a[:k].view(np.uint32))  # sign of -0 preserved


def test_reversal_of_distinct_magnitudes_reverses_mask():
    rng = np.random.default_rng(3)
    a = rng.permutation(np.arange(1, 129)).astype(np.float32) * rng.choice([-1, 1], 128).astype(np.float32)
    _, m1, _, _ = oracle.prune_pack(a, 128, 0.6)
    _, m2, _, _ = oracle.prune_pack(a[::-1].copy(), 128, 0.6)
    assert np.array_equal(_bits(m1, 128), _bits(m2, 128)[::-1])


def test_non_finite_order_by_bit_pattern():
    a = np.array([1.0, np.inf, -np.inf, np.nan, 1e38, -2.0, 0.0, 5.0], dtype=np.float32)
    _, mask, _, k = oracle.prune_pack(a, 8, 0.5)  # keep 4: NaN, +Inf, -Inf, 1e38
    assert k == 4
    assert np.array_equal(np.nonzero(_bits(mask, 8))[0], [1, 2, 3, 4])


def test_ratio_extremes_and_empty():
    a = np.arange(1, 201, dtype=np.float32)
    vals, mask, _, k = oracle.prune_pack(a, 64, 0.0)
    assert k == 200 and np.array_equal(vals, a) and _bits(mask, 200).all()
    vals, mask, _, k = oracle.prune_pack(a, 64, 1.0)
    assert k == 0 and vals.size == 0 and not mask.any()
    vals, mask, _, k = oracle.prune_pack(np.zeros(0, np.float32), 64, 0.5)
    assert k == 0 and mask.size == 0


def test_unpack_roundtrip_and_storage_size():
    rng = np.random.default_rng(11)
    for dtype, s in (("f32", 4), ("bf16", 2)):
        x = rng.standard_normal(5000).astype(np.float32)
        a = x if dtype == "f32" else _bf16(x)
        for r in (0.0, 0.5, 0.9):
            vals, mask, _, k = oracle.prune_pack(a, 512, r)
            dense = oracle.unpack(vals, mask, a.size)
            keep = _bits(mask, a.size)
            expect = np.where(keep, a, np.zeros_like(a))
            assert np.array_equal(dense.view(np.uint8), expect.view(np.uint8))
            # packed bytes = k*s + 8*ceil(n/64): the value vector plus one bit per element (Section 4.2)
            assert vals.nbytes + mask.nbytes == k * s + 8 * ((a.size + 63) // 64)
    # compression closed form (1 - r) + 1/(8 s) when nothing rounds
    n, r = 64 * 1024, 0.75
    vals, mask, _, _ = oracle.prune_pack(rng.standard_normal(n).astype(np.float32), 4096, r)
    assert (vals.nbytes + mask.nbytes) / (4 * n) == pytest.approx((1 - r) + 1 / 32)


def test_group_len_larger_than_n_is_whole_tensor():
    rng = np.random.default_rng(5)
    a = rng.standard_normal(777).astype(np.float32)
    _, m1, _, _ = oracle.prune_pack(a, 777, 0.5)
    _, m2, _, _ = oracle.prune_pack(a, 10**6, 0.5)
    assert np.array_equal(m1, m2)
