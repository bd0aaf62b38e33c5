"""Pins for the oracle's layer scores and pruning ratios (Eq. 5, 6, 7) -- CPU only."""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _examples():
    out = []
    for line in open(os.path.join(GOLDEN, "layer_ratio_examples.txt")):
        if not line.strip() or line.startswith("#"):
            continue
        m, G, p = (np.array(part.split(), dtype=np.float64) for part in line.split("|"))
        out.append((m.astype(np.uint64), G.astype(np.float32), p))
    return out


def test_hand_derived_examples():
    ex = _examples()
    assert len(ex) == 3
    for m, G, p in ex:
        _, _, got = oracle.layer_scores(G, m)
        assert np.allclose(got, p, atol=1e-12)
        assert np.allclose(oracle.layer_ratios(G, m), p.astype(np.float32), atol=1e-7)


def test_intermediate_scores_example1():
    M, I, p = oracle.layer_scores(np.array([1, 2, 4], np.float32), np.array([4, 2, 2], np.uint64))
    assert np.allclose(M, [np.log(2), 2 * np.log(2), 2 * np.log(2)])
    assert np.allclose(I, [0.125, 0.5, 1.0])


def test_invariants():
    rng = np.random.default_rng(2)
    for trial in range(20):
        l = int(rng.integers(2, 60))
        m = rng.integers(1, 10**7, l).astype(np.uint64)
        G = rng.random(l).astype(np.float32) + 1e-3
        M, I, p = oracle.layer_scores(G, m)
        assert (p >= 0).all() and (p <= 1).all()
        assert p[np.argmax(I)] == 0.0  # the most important layer is not pruned (Eq. 7)
        # scaling every G by c > 0 changes nothing (max normalisation)
        _, _, p2 = oracle.layer_scores((G * np.float32(8.0)).astype(np.float32), m)
        assert np.allclose(p, p2, atol=1e-12)
        # the base of the logarithm cancels: recompute Eq. 5-7 with log2 in numpy
        M2 = -np.log2(m.astype(np.float64) / m.astype(np.float64).sum())
        I2 = (M2 / M2.max()) * (G.astype(np.float64) / G.astype(np.float64).max())
        assert np.allclose(p, 1 - I2 / I2.max(), atol=1e-12)
        # scaling every size by a constant changes nothing either (only m_i / sum m enters)
        _, _, p3 = oracle.layer_scores(G, m * np.uint64(3))
        assert np.allclose(p, p3, atol=1e-12)


def test_monotone_in_size_and_gradient():
    """Larger activations get larger ratios, larger gradients smaller ones (end of Section 4.2)."""
    m = np.array([1000, 2000, 4000, 8000], np.uint64)
    G = np.ones(4, np.float32)
    _, _, p = oracle.layer_scores(G, m)
    assert (np.diff(p) > 0).all()
    m = np.full(4, 5000, np.uint64)
    G = np.array([0.1, 0.2, 0.4, 0.8], np.float32)
    _, _, p = oracle.layer_scores(G, m)
    assert (np.diff(p) < 0).all()
    # smaller (deeper) activations score a larger M
    M, _, _ = oracle.layer_scores(np.ones(3, np.float32), np.array([900, 90, 9], np.uint64))
    assert (np.diff(M) > 0).all()


def test_degenerate_cases():
    # one layer: M = -log 1 = 0, 0/0 := 1, p = 0
    assert oracle.layer_ratios(np.array([3.0], np.float32), np.array([10], np.uint64))[0] == 0.0
    # all gradients zero: every layer equally important, p = 0 only where M is maximal
    _, I, p = oracle.layer_scores(np.zeros(3, np.float32), np.array([4, 2, 2], np.uint64))
    assert np.allclose(I, [0.5, 1, 1]) and np.allclose(p, [0.5, 0, 0])
    with pytest.raises(ValueError):
        oracle.layer_scores(np.array([1.0, -1.0], np.float32), np.array([1, 1], np.uint64))
    with pytest.raises(ValueError):
        oracle.layer_scores(np.array([1.0, 1.0], np.float32), np.array([1, 0], np.uint64))
    with pytest.raises(ValueError):
        oracle.layer_scores(np.array([1.0, np.nan], np.float32), np.array([1, 1], np.uint64))


def test_affine_map_into_interval():
    m, G, p = _examples()[0]
    r = oracle.layer_ratios(G, m, 0.3, 0.9)
    assert np.allclose(r, 0.3 + 0.6 * p, atol=1e-7)
    assert r.dtype == np.float32
    with pytest.raises(ValueError):
        oracle.layer_ratios(G, m, 0.9, 0.3)
