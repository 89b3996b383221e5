"""Pins for a draft model with its own output embedding (Ablation 3, "A / B" = draft model A,
verify model B).  Theorem 1 holds for any draft law rho, so what the paper fixes is: the emitted
token still follows the TARGET law, the draft token follows the law of the draft model's own head,
acceptance has probability sum_v min(p_v, q_v) with that q, and one shared head is the special case."""
import numpy as np
import scipy.special
from scipy import stats

from oracle import fef_oracle as O


def _chi2_p(counts, probs):
    n = counts.sum()
    return stats.chi2.sf(np.sum((counts - n * probs) ** 2 / (n * probs)), len(probs) - 1)


def _two_heads(V, d, K, seed):
    rng = np.random.default_rng(seed)
    s = 2.0 / (0.02 * np.sqrt(d))
    W_t = rng.normal(size=(V, d)) * 0.02
    W_d = 0.8 * W_t + 0.6 * rng.normal(size=(V, d)) * 0.02      # a related but different head
    hd = rng.normal(size=(K, d)) * s
    ht = 0.7 * hd + np.sqrt(1 - 0.49) * rng.normal(size=(K, d)) * s
    return W_t, W_d, hd, ht


def test_same_head_is_the_default():
    W_t, W_d, hd, ht = _two_heads(12, 16, 3, 0)
    a = O.verify_step(hd[None], ht[None], W_t, 3, 4, 5, return_logits=True)
    b = O.verify_step(hd[None], ht[None], W_t, 3, 4, 5, return_logits=True, W_draft=W_t)
    for f in ("tokens", "accept_len", "remask", "alpha", "logits", "lse", "draft_tokens"):
        assert np.array_equal(getattr(a, f), getattr(b, f)), f


def test_laws_come_from_the_two_heads():
    """Library softmax of the two projections, written out: q from (h_draft, W_draft), p from (h_target, W)."""
    W_t, W_d, hd, ht = _two_heads(10, 16, 2, 1)
    tau = 0.7
    r = O.verify_step(hd[None], ht[None], W_t, 2, 2, 3, temperature=tau, return_logits=True, W_draft=W_d)
    Lq = np.einsum("kd,vd->kv", hd, W_d) / tau
    Lp = np.einsum("kd,vd->kv", ht, W_t) / tau
    assert np.allclose(r.logits[0, 0], Lq, atol=1e-12) and np.allclose(r.logits[1, 0], Lp, atol=1e-12)
    q, p = scipy.special.softmax(Lq, -1), scipy.special.softmax(Lp, -1)
    assert np.allclose(r.alpha[0], np.minimum(p, q).sum(-1), atol=1e-12)
    assert np.allclose(r.lse[0, 0], scipy.special.logsumexp(Lq, -1), atol=1e-12)
    # with the heads swapped the draft logits change and the target logits do not
    r2 = O.verify_step(hd[None], ht[None], W_t, 2, 2, 3, temperature=tau, return_logits=True, W_draft=W_t)
    assert np.array_equal(r.logits[1], r2.logits[1]) and not np.allclose(r.logits[0], r2.logits[0])


def test_emitted_law_is_the_target_law_whatever_the_draft_head():
    V, d, n = 8, 16, 400_000
    W_t, W_d, hd, ht = _two_heads(V, d, 1, 2)
    q = scipy.special.softmax(hd @ W_d.T, -1)[0]
    p = scipy.special.softmax(ht @ W_t.T, -1)[0]
    q_shared = scipy.special.softmax(hd @ W_t.T, -1)[0]
    alpha = np.minimum(p, q).sum()
    assert 0.2 < alpha < 0.95 and np.abs(q - q_shared).max() > 0.02
    res = O.verify_step(np.broadcast_to(hd, (n, 1, d)), np.broadcast_to(ht, (n, 1, d)), W_t, K=1, block=1,
                        seed=77, W_draft=W_d)
    assert _chi2_p(np.bincount(res.tokens[:, 0], minlength=V), p) > 1e-3            # Theorem 1
    drafted = np.bincount(res.draft_tokens[:, 0], minlength=V)
    assert _chi2_p(drafted, q) > 1e-3 and _chi2_p(drafted, q_shared) < 1e-6          # the draft model's own law
    acc = (res.accept_len == 1).mean()
    assert abs(acc - alpha) < 4 * np.sqrt(alpha * (1 - alpha) / n)
