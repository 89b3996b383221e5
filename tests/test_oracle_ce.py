"""Pins for the cross-entropy oracle (Algorithm 1's token-level loss through the vocabulary head):
library log-softmax, closed forms, brute force, and the link to the decoding laws."""
import math

import numpy as np
import scipy.special

from oracle import ce_oracle as C
from oracle import fef_oracle as O


def _inst(seed, R=9, d=20, V=33, scale=3.0):
    rng = np.random.default_rng(seed)
    W = rng.normal(size=(V, d)) * 0.02
    h = rng.normal(size=(R, d)) * scale / (0.02 * np.sqrt(d))
    y = rng.integers(0, V, size=R)
    return h, W, y


def test_against_library_log_softmax_and_sum():
    for seed, tau in [(0, 1.0), (1, 0.5), (2, 2.0)]:
        h, W, y = _inst(seed)
        ce, loss = C.cross_entropy(h, W, y, temperature=tau)
        want = -scipy.special.log_softmax(h @ W.T / tau, axis=-1)[np.arange(len(y)), y]
        assert np.allclose(ce, want, rtol=1e-13, atol=1e-13)
        assert abs(loss - want.sum()) < 1e-11
        assert np.all(ce > 0)


def test_closed_forms():
    h, W, y = _inst(3, R=4, V=17)
    ce, _ = C.cross_entropy(np.zeros_like(h), W, y)          # uniform law: CE = log V
    assert np.allclose(ce, math.log(17))
    W2 = np.zeros((5, 3)); W2[2] = [1.0, 0, 0]
    hh = np.array([[50.0, 0, 0]])                             # token 2 dominates by 50 nats
    assert C.cross_entropy(hh, W2, [2])[0][0] < 1e-20 + 4 * math.exp(-50) * 1.01
    assert abs(C.cross_entropy(hh, W2, [0])[0][0] - (50 + math.log1p(4 * math.exp(-50)))) < 1e-12
    # shifting every logit of a row (adding a vector orthogonal to nothing: a constant column) changes nothing
    h3, W3, y3 = _inst(4)
    W3s = np.concatenate([W3, np.ones((W3.shape[0], 1))], axis=1)
    h3s = np.concatenate([h3, 7.5 * np.ones((h3.shape[0], 1))], axis=1)
    assert np.allclose(C.cross_entropy(h3, W3, y3)[0], C.cross_entropy(h3s, W3s, y3)[0], rtol=1e-12)


def test_brute_force_and_skipped_rows():
    h, W, y = _inst(5, R=5, d=6, V=7)
    y = y.copy(); y[3] = -1
    ce, loss = C.cross_entropy(h, W, y)
    for m in range(5):
        if y[m] < 0:
            assert ce[m] == 0.0
            continue
        logits = [sum(h[m][k] * W[v][k] for k in range(6)) for v in range(7)]
        z = sum(math.exp(l) for l in logits)
        assert abs(ce[m] - (math.log(z) - logits[y[m]])) < 1e-12
    assert abs(loss - ce.sum()) < 1e-12


def test_is_minus_log_of_the_decoding_law():
    """The predictor of Algorithm 1 is the target law of Algorithm 2: CE = -log pi(token)."""
    h, W, y = _inst(6)
    pi, _ = O.law(O.head_logits(h, W, 1.0))
    ce, _ = C.cross_entropy(h, W, y)
    assert np.allclose(np.exp(-ce), pi[np.arange(len(y)), y], rtol=1e-12)
    # expected CE under labels drawn from the law itself is its entropy
    ent = -(pi * np.log(pi)).sum(-1)
    exp_ce = np.array([sum(pi[m, v] * C.cross_entropy(h[m:m + 1], W, [v])[0][0] for v in range(W.shape[0]))
                       for m in range(h.shape[0])])
    assert np.allclose(exp_ce, ent, rtol=1e-11)
