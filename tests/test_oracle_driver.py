"""Pins for the oracle's Algorithm 2 outer loops (oracle/driver.py): pass structure, LowConf
budget, round counts, and agreement with chaining verify_step by hand."""
import math

import numpy as np

from oracle import driver as D
from oracle import fef_oracle as O


def _setup(seed, B=3, K=4, d=32, V=24, rho=0.8):
    rng = np.random.default_rng(seed)
    W = rng.normal(size=(V, d)) * 0.02
    s = 2.0 / (0.02 * np.sqrt(d))
    cache = {}

    def hidden(r):
        if r not in cache:
            g = np.random.default_rng(1000 * seed + r)
            hd = g.normal(size=(B, K, d)) * s
            cache[r] = (hd, rho * hd + np.sqrt(1 - rho ** 2) * g.normal(size=(B, K, d)) * s)
        return cache[r]
    return W, hidden


def test_pass_structure_and_budgets():
    B, K, block = 3, 4, 12
    W, hidden = _setup(1, B=B, K=K)
    for n_pass, n_rm in [(1, 5), (2, 5), (3, -1), (3, 0), (2, 100)]:
        res = D.decode_block(hidden, W, B, K, block, seed=7, n_pass=n_pass, n_rm=n_rm)
        budget = block // 2 if n_rm < 0 else min(n_rm, block)
        assert np.all(res.X >= 0)                      # no MASK left after the last pass
        for b in range(B):
            cp, rp = res.committed_per_pass[b], res.rounds_per_pass[b]
            assert len(cp) == n_pass and cp[0] == block     # pass 0 resolves the whole block
            want = budget
            for s in range(1, n_pass):
                assert cp[s] == want                        # pass s re-resolves LowConf's selection
                want = min(budget, cp[s])                   # candidates of the next LowConf: C^(s) only
            for s in range(n_pass):
                assert rp[s] >= math.ceil(cp[s] / K)        # at most k positions per round
                assert rp[s] <= cp[s]                       # at least one position per round
            assert res.rounds[b] == sum(rp)


def test_single_pass_equals_hand_chained_rounds():
    B, K, block = 2, 4, 10
    W, hidden = _setup(2, B=B, K=K)
    res = D.decode_block(hidden, W, B, K, block, seed=3, n_pass=1, pos_base=40, step_base=5, seq_base=9)
    for b in range(B):
        mask = np.ones((1, block), np.uint8)
        X = np.full(block, -1)
        r = 0
        while mask.any():
            hd, ht = hidden(r)
            st = O.verify_step(hd[b:b + 1], ht[b:b + 1], W, K, block, 3, step=5 + r, seq_base=9 + b, pos_base=40,
                               final_pass=True, mask_in=mask)
            for m in range(st.committed[0]):
                X[st.slot_pos[0, m]] = st.tokens[0, m]
            mask = st.remask
            r += 1
        assert r == res.rounds[b]
        assert np.array_equal(X, res.X[b])


def test_rounds_follow_expected_committed_length():
    """Rounds per pass ~ L / E[C_k] (Theorem 2) when every slot shares one acceptance probability."""
    B, K, block, d, V = 400, 4, 32, 16, 8
    rng = np.random.default_rng(5)
    W = rng.normal(size=(V, d)) * 0.02
    s = 1.5 / (0.02 * np.sqrt(d))
    hd1 = rng.normal(size=(1, 1, d)) * s
    ht1 = 0.8 * hd1 + 0.6 * rng.normal(size=(1, 1, d)) * s
    hd = np.broadcast_to(hd1, (B, K, d)); ht = np.broadcast_to(ht1, (B, K, d))
    res = D.decode_block(lambda r: (hd, ht), W, B, K, block, seed=11, n_pass=1)
    alpha = res.alpha_mean.mean()
    per_round = block / res.rounds.mean()
    # the last window of a block is shorter than k, so the mean lies a little below E[C_k]
    assert 0.85 * O.expected_committed_iid(alpha, K) < per_round <= O.expected_committed_iid(alpha, K) + 0.05
