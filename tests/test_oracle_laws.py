"""Pins for the oracle's building blocks: head projection, softmax / log-sum-exp, the
residual law and its identities (proof of Theorem 1, residual-distribution equation),
inverse-CDF sampling, window selection and LowConf."""
import itertools

import numpy as np
import pytest
import scipy.special

from oracle import fef_oracle as O


def _laws(rng, B, V, scale=2.0):
    p = scipy.special.softmax(rng.normal(size=(B, V)) * scale, axis=-1)
    q = scipy.special.softmax(rng.normal(size=(B, V)) * scale, axis=-1)
    return p, q


def test_head_logits_brute_force():
    rng = np.random.default_rng(0)
    h = rng.normal(size=(3, 5))
    W = rng.normal(size=(7, 5))            # V=7 != d=5 so a transposed operand cannot pass
    L = O.head_logits(h, W, 0.5)
    assert L.shape == (3, 7)
    for r in range(3):
        for v in range(7):
            s = 0.0
            for k in range(5):
                s += h[r, k] * W[v, k]
            assert L[r, v] == pytest.approx(s / 0.5, rel=1e-13, abs=1e-13)


def test_law_matches_library_softmax_and_logsumexp():
    rng = np.random.default_rng(1)
    L = rng.normal(size=(4, 1000)) * 5 + 300.0     # large offset: needs the max shift
    p, lse = O.law(L)
    assert np.allclose(lse, scipy.special.logsumexp(L, axis=-1), rtol=0, atol=1e-10)
    assert np.allclose(p, scipy.special.softmax(L, axis=-1), rtol=1e-12, atol=0)
    assert np.all(np.abs(p.sum(-1) - 1) < 1e-12)
    assert np.all(np.isfinite(p))


def test_residual_identities():
    rng = np.random.default_rng(2)
    p, q = _laws(rng, 16, 32)
    r, Z = O.residual_law(p, q)
    alpha = np.minimum(p, q).sum(-1)
    # residual-distribution equation: normaliser 1 - sum min = sum [p-q]_+ = half the L1 distance
    assert np.allclose(Z, 1 - alpha, atol=1e-12)
    assert np.allclose(Z, 0.5 * np.abs(p - q).sum(-1), atol=1e-12)
    pi_prime = r / Z[:, None]
    assert np.allclose(pi_prime.sum(-1), 1, atol=1e-12)
    assert np.all(pi_prime >= 0)
    # support: the residual vanishes exactly where the draft over-proposes
    assert np.all((pi_prime > 0) == (p > q))
    # one-step identity of Theorem 1's proof: min(p,q) + (1 - sum min) pi' = p for every token
    assert np.allclose(np.minimum(p, q) + Z[:, None] * pi_prime, p, atol=1e-12)
    # acceptance mass per token: q min(1, p/q) = min(p, q), summed = alpha
    assert np.allclose((q * np.minimum(1, p / q)).sum(-1), alpha, atol=1e-12)
    # a sign slip (q - p) would give a different law whenever p != q
    assert not np.allclose(np.maximum(q - p, 0), r)


def test_residual_of_identical_laws_is_zero():
    rng = np.random.default_rng(3)
    p, _ = _laws(rng, 2, 8)
    r, Z = O.residual_law(p, p)
    assert np.all(r == 0) and np.all(Z == 0)


def _first_reaching(mass, target):
    s = 0.0
    for v, m in enumerate(mass):
        s += m
        if s >= target:
            return v
    return max(v for v, m in enumerate(mass) if m > 0)


def test_inverse_cdf_brute_force_and_library():
    rng = np.random.default_rng(4)
    mass = rng.random((200, 13))
    mass[rng.random((200, 13)) < 0.3] = 0.0       # zero-mass tokens must never be selected
    mass[:, 5] += 0.1
    mass /= mass.sum(-1, keepdims=True)
    u = rng.random(200)
    idx, gap = O.inverse_cdf(mass, u)
    for i in range(200):
        assert idx[i] == _first_reaching(mass[i], u[i])
        assert mass[i, idx[i]] > 0
        cdf = np.cumsum(mass[i])
        assert idx[i] == np.searchsorted(cdf, u[i], side="left")
        edges = [abs(cdf[idx[i]] - u[i])] if idx[i] < 12 else []
        if idx[i] > 0:
            edges.append(abs(u[i] - cdf[idx[i] - 1]))
        assert gap[i] == pytest.approx(min(edges)) if edges else np.isinf(gap[i])


def test_inverse_cdf_edges():
    mass = np.array([[0.25, 0.25, 0.5, 0.0]])
    assert O.inverse_cdf(mass, np.array([0.25]))[0][0] == 0      # ">=": boundary belongs below
    assert O.inverse_cdf(mass, np.array([0.2500001]))[0][0] == 1
    assert O.inverse_cdf(mass, np.array([1.0]))[0][0] == 2       # never the empty last token
    assert O.inverse_cdf(mass, np.array([1.5]))[0][0] == 2       # unreachable target -> last positive
    assert O.inverse_cdf(mass, np.array([1e-30]))[0][0] == 0


def test_inverse_cdf_distribution():
    rng = np.random.default_rng(5)
    mass = scipy.special.softmax(rng.normal(size=8) * 1.5)
    n = 200_000
    idx, _ = O.inverse_cdf(np.broadcast_to(mass, (n, 8)), (np.arange(n) + 0.5) / n)
    counts = np.bincount(idx, minlength=8)
    assert np.all(np.abs(counts / n - mass) < 2 / n + 1e-12)     # stratified uniforms: exact up to 1 count per edge


def test_window_slots():
    mask = np.array([[0, 1, 1, 0, 1, 1, 1, 0],
                     [0, 0, 0, 0, 0, 1, 0, 1],
                     [0, 0, 0, 0, 0, 0, 0, 0]], np.uint8)
    pos, win = O.window_slots(mask, 4)
    assert win.tolist() == [4, 2, 0]
    assert pos.tolist() == [[1, 2, 4, 5], [5, 7, -1, -1], [-1, -1, -1, -1]]


def test_low_confidence_brute_force():
    rng = np.random.default_rng(6)
    for trial in range(200):
        n = int(rng.integers(1, 9))
        conf = np.round(rng.random(n), 1)              # coarse values -> many ties
        cand = (rng.random(n) < 0.7).astype(np.uint8)
        n_rm = int(rng.integers(0, n + 2))
        sel, gap = O.low_confidence(conf, cand, n_rm)
        c = [i for i in range(n) if cand[i]]
        want = sorted(c, key=lambda i: (conf[i], i))[:n_rm]
        assert sel.tolist() == want
        assert len(sel) == min(n_rm, len(c))
        # brute force over subsets: no unselected candidate beats a selected one
        for i, j in itertools.product(sel.tolist(), set(c) - set(sel.tolist())):
            assert (conf[i], i) < (conf[j], j)
        if 0 < len(sel) < len(c):
            assert gap == pytest.approx(min(conf[j] for j in set(c) - set(sel.tolist())) - max(conf[i] for i in sel))
        else:
            assert np.isinf(gap)
