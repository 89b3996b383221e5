"""Pins for the baseline step oracle (LLaDA's parallel prediction with top-n confidence transfer):
brute force, library softmax, the sampling law, and the special cases n = 1 and n >= window."""
import numpy as np
import scipy.special
from scipy import stats

from oracle import fef_oracle as O
from oracle import llada_oracle as LO


def _inst(seed, B=5, K=6, d=16, V=20, scale=2.5):
    rng = np.random.default_rng(seed)
    W = rng.normal(size=(V, d)) * 0.02
    h = rng.normal(size=(B, K, d)) * scale / (0.02 * np.sqrt(d))
    return h, W


def test_brute_force_selection_and_confidences():
    h, W = _inst(1)
    B, K = h.shape[:2]
    block = 8
    mask = np.ones((B, block), np.uint8); mask[0, [1, 5]] = 0; mask[1, :] = 0; mask[2, 3:] = 0
    conf0 = np.full((B, block), 0.123)
    for n in (1, 2, 3, 50):
        for greedy in (False, True):
            r = LO.topn_step(h, W, K, block, seed=4, n_transfer=n, mask_in=mask, conf=conf0, greedy=greedy, temperature=0.9)
            for b in range(B):
                pos = [i for i in range(block) if mask[b, i]][:K]
                assert r.window[b] == len(pos) and r.slot_pos[b, :len(pos)].tolist() == pos
                pis = [scipy.special.softmax(h[b, m] @ W.T / 0.9) for m in range(len(pos))]
                xs = r.drawn[b, :len(pos)]
                if greedy:
                    assert xs.tolist() == [int(np.argmax(p)) for p in pis]
                cs = [pis[m][xs[m]] for m in range(len(pos))]
                assert np.allclose(r.slot_conf[b, :len(pos)], cs, rtol=1e-12)
                # brute force: repeatedly take the most confident remaining slot (lower position on ties)
                left = list(range(len(pos)))
                take = []
                for _ in range(min(n, len(pos))):
                    best = max(left, key=lambda m: (cs[m], -pos[m]))
                    take.append(best); left.remove(best)
                want_tok = [-1] * K
                for m in take:
                    want_tok[m] = int(xs[m])
                assert r.tokens[b].tolist() == want_tok and r.committed[b] == len(take)
                want_mask = mask[b].copy()
                want_mask[[pos[m] for m in take]] = 0
                assert np.array_equal(r.remask[b], want_mask)
                for i in range(block):
                    if i in [pos[m] for m in take]:
                        assert abs(r.conf[b, i] - cs[take[[pos[m] for m in take].index(i)]]) < 1e-12
                    else:
                        assert r.conf[b, i] == 0.123


def test_drawn_tokens_follow_the_law():
    rng = np.random.default_rng(5)
    V, d = 6, 8
    W = rng.normal(size=(V, d)) * 0.02
    hrow = rng.normal(size=d) * 2.0 / (0.02 * np.sqrt(d))
    p = scipy.special.softmax(hrow @ W.T)
    B = 20000
    h = np.broadcast_to(hrow, (B, 1, d)).copy()
    r = LO.topn_step(h, W, 1, 1, seed=9, n_transfer=1)
    counts = np.bincount(r.tokens[:, 0], minlength=V)
    chi2 = ((counts - B * p) ** 2 / (B * p)).sum()
    assert stats.chi2.sf(chi2, V - 1) > 1e-4
    # the draw is the speculative step's draft draw at the same counters (same law, same stream)
    s = O.verify_step(h[:50], h[:50], W, 1, 1, seed=9)
    assert np.array_equal(s.draft_tokens[:, 0], r.drawn[:50, 0])


def test_n_at_least_window_commits_everything_and_n1_commits_the_most_confident():
    h, W = _inst(3, B=4, K=5)
    full = LO.topn_step(h, W, 5, 5, seed=2, n_transfer=5)
    assert np.all(full.remask == 0) and np.array_equal(full.tokens, full.drawn)
    one = LO.topn_step(h, W, 5, 5, seed=2, n_transfer=1)
    assert np.all(one.committed == 1) and np.all(one.remask.sum(1) == 4)
    best = np.argmax(full.slot_conf, axis=1)
    assert np.all(one.tokens[np.arange(4), best] == full.drawn[np.arange(4), best])
    assert np.all((one.tokens >= 0).sum(1) == 1)
    # chaining steps with n = 2 resolves a block of 5 in 3 steps, never committing a position twice
    mask = np.ones((4, 5), np.uint8)
    for step in range(3):
        r = LO.topn_step(h, W, 5, 5, seed=2, n_transfer=2, mask_in=mask, step=step)
        assert np.all(r.remask <= mask) and np.all(mask.sum(1) - r.remask.sum(1) == r.committed)
        mask = r.remask
    assert mask.sum() == 0
