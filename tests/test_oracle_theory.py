"""Cross-check of the oracle's Theorem 2 / Corollary 2 functions and of its accept_len
semantics against numbers the paper prints (Tables 1, 3, 4, 5; fixture with citations in
tests/golden/paper_tables_speed_acceptance.txt).

Reading tested here: Table 4's "Acceptance" is accepted drafts / proposed drafts per round,
E[a]/k with E[a] = sum_{l=1..k} alpha^l; the committed count C_k includes the corrected
position and has no extra token after a full window; with draft = target model
(c_rho ~ c_pi) the speed-up over prefix-conditioned decoding without speculation is
E[C_k]/2.  Then (speed with SD)/(speed without SD) must equal E[C_k]/2 with alpha backed out
of the printed acceptance."""
import os

import numpy as np
import pytest
from scipy import optimize

from oracle import fef_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_tables_speed_acceptance.txt")


def _load():
    bench, window, nosd = {}, {}, {}
    with open(GOLDEN) as f:
        for line in f:
            t = line.split("#")[0].split()
            if not t:
                continue
            if t[0] == "window":
                window[int(t[1])] = float(t[2])
            elif t[0] == "nosd":
                nosd[int(t[1])] = float(t[2])
            else:
                bench[t[0]] = tuple(float(x) for x in t[1:4])
    return bench, window, nosd


def _alpha_from_acceptance(acc, k):
    f = lambda a: (O.expected_committed_iid(a, k + 1) - 1.0) / k - acc   # sum_{l=1..k} a^l / k
    return optimize.brentq(f, 1e-9, 1 - 1e-12)


def test_speedup_ratio_matches_expected_committed_over_two():
    bench, window, _ = _load()
    assert len(bench) == 4
    for name, (acc_pct, with_sd, without_sd) in bench.items():
        alpha = _alpha_from_acceptance(acc_pct / 100.0, 16)
        predicted = O.acceleration_ratio(alpha, 16)            # c_rho = c_pi
        measured = with_sd / without_sd
        assert predicted == pytest.approx(measured, rel=0.05), name
        # a bonus token after a full window (classic speculative decoding) would not fit:
        # E[C]+alpha^16 over 2 passes
        assert 0.5 * (O.expected_committed_iid(alpha, 16)) < 16 / 2


def test_window_ablation_matches_with_the_same_alpha():
    bench, window, _ = _load()
    alpha = _alpha_from_acceptance(bench["GSM8K"][0] / 100.0, 16)
    base = bench["GSM8K"][2]
    for k, speed in window.items():
        assert O.acceleration_ratio(alpha, k) == pytest.approx(speed / base, rel=0.05), k


def test_resampling_budget_reading_half_block():
    """Without speculation one position costs one target pass, so N_step passes that each
    re-resolve half of the positions cost 1 + (N_step-1)/2 relative to one-token-per-step
    decoding: the printed 0.67x and 0.40x."""
    _, _, nosd = _load()
    for n_step, speed in nosd.items():
        assert 1.0 / (1.0 + 0.5 * (n_step - 1)) == pytest.approx(speed, abs=0.01)


def test_oracle_accept_rate_statistic_matches_reading():
    """Simulated rounds: accepted/proposed equals sum_{l=1..k} alpha^l / k."""
    rng = np.random.default_rng(0)
    V, d, K, n = 8, 16, 16, 50_000
    W = rng.normal(size=(V, d)) * 0.02
    s = 1.0 / (0.02 * np.sqrt(d))
    hd = rng.normal(size=(1, d)) * s
    ht = 0.9 * hd + np.sqrt(0.19) * rng.normal(size=(1, d)) * s
    H = np.broadcast_to(hd, (n, K, d)); T = np.broadcast_to(ht, (n, K, d))
    res = O.verify_step(H, T, W, K=K, block=K, seed=77)
    alpha = res.alpha[0, 0]
    want = (O.expected_committed_iid(alpha, K + 1) - 1.0) / K
    got = res.accept_len.mean() / K
    assert abs(got - want) < 4 * res.accept_len.std() / K / np.sqrt(n)
