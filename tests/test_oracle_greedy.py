"""Pins for the oracle's greedy variant: the zero-temperature limit of Algorithm 2's laws (point
masses at the arg max), checked against the sampled oracle at a tiny temperature, brute force,
library softmax, Theorem 2 with acceptance probabilities in {0, 1}, and tie handling."""
import numpy as np
import scipy.special

from oracle import fef_oracle as O


def _inst(seed, B=6, K=4, d=24, V=40, rho=0.7, scale=3.0):
    rng = np.random.default_rng(seed)
    W = rng.normal(size=(V, d)) * 0.02
    s = scale / (0.02 * np.sqrt(d))
    hd = rng.normal(size=(B, K, d)) * s
    ht = rho * hd + np.sqrt(1 - rho ** 2) * rng.normal(size=(B, K, d)) * s
    return hd, ht, W


def test_greedy_is_the_zero_temperature_limit_of_the_sampled_step():
    """With the logits fixed and tau -> 0 the sampled round commits the greedy tokens whatever
    the uniforms are (checked where every arg max is clear of its runner-up)."""
    checked = 0
    for seed in range(12):
        hd, ht, W = _inst(seed)
        B, K = hd.shape[:2]
        g = O.verify_step(hd, ht, W, K, 8, seed=seed, greedy=True)
        clear = g.argmax_gap.min(axis=(0, 2)) > 0.05
        for s2 in (1, 99):
            cold = O.verify_step(hd, ht, W, K, 8, seed=s2, step=seed, temperature=1e-3)
            assert np.array_equal(cold.tokens[clear], g.tokens[clear])
            assert np.array_equal(cold.accept_len[clear], g.accept_len[clear])
            assert np.array_equal(cold.remask[clear], g.remask[clear])
        checked += int(clear.sum())
    assert checked > 40


def test_greedy_brute_force_tokens_confidences_and_theorem_2_with_binary_alpha():
    hd, ht, W = _inst(3, B=8, K=3, V=31, rho=0.98)
    B, K = hd.shape[:2]
    tau = 0.7
    r = O.verify_step(hd, ht, W, K, 12, seed=0, temperature=tau, greedy=True)
    rejected = 0
    for b in range(B):
        Lq = [[sum(hd[b, m, k] * W[v, k] for k in range(W.shape[1])) for v in range(W.shape[0])] for m in range(K)]
        Lp = [[sum(ht[b, m, k] * W[v, k] for k in range(W.shape[1])) for v in range(W.shape[0])] for m in range(K)]
        aq = [max(range(len(row)), key=lambda v: (row[v], -v)) for row in Lq]
        ap = [max(range(len(row)), key=lambda v: (row[v], -v)) for row in Lp]
        a = next((m for m in range(K) if aq[m] != ap[m]), K)        # first slot whose arg maxes differ
        assert r.accept_len[b] == a
        assert r.committed[b] == min(a + 1, K)                      # Theorem 2 with alpha in {0, 1}
        want = [aq[m] for m in range(a)] + ([ap[a]] if a < K else [])
        assert r.tokens[b, :len(want)].tolist() == want and np.all(r.tokens[b, len(want):] == -1)
        assert r.draft_tokens[b].tolist() == aq
        for m, tok in enumerate(want):                               # confidence = pi_tau(token)
            pi = scipy.special.softmax(np.array(Lp[m]) / tau)
            assert abs(r.conf[b, r.slot_pos[b, m]] - pi[tok]) < 1e-12
        rejected += int(a < K)
    assert 0 < rejected < B


def test_greedy_draws_no_uniform_and_accepts_identical_models():
    hd, ht, W = _inst(5)
    K = hd.shape[1]
    a = O.verify_step(hd, ht, W, K, 8, seed=1, step=0, greedy=True)
    b = O.verify_step(hd, ht, W, K, 8, seed=2 ** 40 + 7, step=55, seq_base=9, pos_base=300, greedy=True)
    for f in ("tokens", "accept_len", "remask", "conf", "draft_tokens"):
        assert np.array_equal(getattr(a, f), getattr(b, f))
    same = O.verify_step(hd, hd, W, K, 8, seed=1, greedy=True)
    assert np.all(same.accept_len == K) and np.array_equal(same.tokens, same.draft_tokens)


def test_greedy_ties_take_the_lowest_token_id_and_supplied_drafts_are_compared():
    hd, ht, W = _inst(7, B=3, K=2, V=12)
    hd[...] = 0; ht[...] = 0                      # all logits equal (zero): every token ties
    r = O.verify_step(hd, ht, W, 2, 4, seed=0, greedy=True)
    assert np.all(r.draft_tokens == 0) and np.all(r.tokens == 0) and np.all(r.accept_len == 2)
    assert np.all(r.argmax_gap == 0)
    hd, ht, W = _inst(7, B=3, K=2, V=12)
    W[9] = 3 * W[4]                               # make 4 and 9 the two largest ...
    Lq = np.einsum("bkd,vd->bkv", hd, W)
    lead = np.argmax(Lq, axis=-1)
    W[9] = W[4]                                   # ... and then an exact tie between them
    r = O.verify_step(hd, hd, W, 2, 4, seed=0, greedy=True)
    tied = np.isin(lead, (4, 9)) & (np.argmax(np.einsum("bkd,vd->bkv", hd, W), axis=-1) == 4)
    assert np.all(r.draft_tokens[tied] == 4) and not np.any(r.draft_tokens == 9)
    hd2, ht2, W2 = _inst(8, B=4, K=3, V=20)
    g = O.verify_step(hd2, ht2, W2, 3, 6, seed=0, greedy=True)
    top = np.argmax(np.einsum("bkd,vd->bkv", ht2, W2), axis=-1)
    drafts = top.copy()
    drafts[1, 1] = (drafts[1, 1] + 1) % 20        # one wrong draft: rejected there, corrected to arg max pi
    s = O.verify_step(hd2, ht2, W2, 3, 6, seed=0, greedy=True, draft_tokens=drafts)
    assert s.accept_len.tolist() == [3, 1, 3, 3]
    assert s.tokens[1].tolist() == [top[1, 0], top[1, 1], -1]
    assert g.tokens.shape == s.tokens.shape
