"""Pins for the oracle's stochastic re-corruption (Algorithm 2, "Re-corrupt X^i ~ q(X_t^i |
X_0^i)" with the absorbing forward kernel of D3PM): what the kernel's definition fixes is that
each selected position becomes MASK independently with probability 1 - alpha-bar_t and keeps
its token otherwise; everything below follows from that, none of it from the oracle's code."""
import numpy as np
from scipy import stats

from oracle import driver as D
from oracle import fef_oracle as O
from oracle import philox


def test_probability_one_is_the_always_mask_reading():
    sel = np.array([5, 1, 9])
    assert np.array_equal(O.recorrupt(sel, 1.0, 3, 0, 0, 0), sel)
    assert O.recorrupt(np.array([], np.int64), 0.3, 3, 0, 0, 0).size == 0


def test_marginal_is_bernoulli_and_positions_are_independent():
    """Absorbing kernel: P(MASK) = prob for each position, independently of the others."""
    n_pos, trials = 8, 6000
    sel = np.arange(n_pos)
    for prob in (0.25, 0.5, 0.9):
        hits = np.zeros((trials, n_pos), bool)
        for t in range(trials):
            hits[t, O.recorrupt(sel, prob, seed=11, pos_base=100, step=t, sequence=t % 7)] = True
        freq = hits.mean(0)
        sigma = np.sqrt(prob * (1 - prob) / trials)
        assert np.all(np.abs(freq - prob) < 4.5 * sigma), (prob, freq)
        # pairwise independence: joint frequency of two positions = prob^2
        joint = (hits[:, :, None] & hits[:, None, :]).mean(0)
        off = joint[~np.eye(n_pos, dtype=bool)]
        s2 = np.sqrt(prob ** 2 * (1 - prob ** 2) / trials)
        assert np.all(np.abs(off - prob ** 2) < 4.5 * s2)
        # the number masked per trial is Binomial(n_pos, prob)
        counts = np.bincount(hits.sum(1), minlength=n_pos + 1)
        expect = stats.binom.pmf(np.arange(n_pos + 1), n_pos, prob) * trials
        keep = expect > 5
        chi2 = ((counts[keep] - expect[keep]) ** 2 / expect[keep]).sum()
        assert stats.chi2.sf(chi2, keep.sum() - 1) > 1e-4


def test_exact_probability_on_the_uniform_grid():
    """The 2^23 uniforms are (j + 1/2) 2^-23; a threshold p = m 2^-23 must be undercut by
    exactly m of them, so P(MASK) = p with no bias.  Checked on the decision itself by
    feeding positions whose uniforms are known from the generator."""
    pos = np.arange(4096)
    u = philox.uniform(9, 50 + pos, 2, 3, 3)       # stream 3 = re-corruption
    for p in (0.125, 0.5, 0.75):
        got = O.recorrupt(pos, p, 9, 50, 2, 3)
        assert np.array_equal(got, pos[u < p])
        j = np.arange(2 ** 12) * 2 ** 11            # a coarse sub-grid of the 2^23 values
        assert ((j + 0.5) * 2.0 ** -23 < p).mean() == p


def test_masks_are_nested_in_the_probability_and_use_their_own_stream():
    sel = np.arange(64)
    prev = set()
    for prob in (0.1, 0.3, 0.6, 0.95, 1.0):
        cur = set(O.recorrupt(sel, prob, 5, 0, 4, 1).tolist())
        assert prev <= cur                          # same uniform, growing threshold
        prev = cur
    # the draw does not reuse the accept / draft / residual uniforms of the same counter
    u3 = philox.uniform(5, sel, 4, 1, philox.STREAM_RECORRUPT)
    for other in (philox.STREAM_DRAFT, philox.STREAM_ACCEPT, philox.STREAM_RESIDUAL):
        assert not np.any(u3 == philox.uniform(5, sel, 4, 1, other))
    # and it is keyed by absolute position, step and sequence
    a = O.recorrupt(sel, 0.5, 5, 0, 4, 1)
    assert not np.array_equal(a, O.recorrupt(sel, 0.5, 5, 0, 5, 1))
    assert not np.array_equal(a, O.recorrupt(sel, 0.5, 5, 0, 4, 2))
    assert np.array_equal(O.recorrupt(sel + 7, 0.5, 5, 0, 4, 1), O.recorrupt(sel, 0.5, 5, 7, 4, 1) + 7)


def _laws(seed, B, K, d, V, rho=0.8):
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


def test_step_remasks_a_subset_of_the_low_confidence_selection():
    B, K, block, V, d = 5, 4, 4, 24, 16
    W, hidden = _laws(4, B, K, d, V)
    hd, ht = hidden(0)
    # identical laws accept the whole window, so one round resolves the block and LowConf fires
    full = O.verify_step(hd, hd, W, K, block, 3, n_rm=3)
    assert np.all(full.remask.sum(1) == 3)
    total = 0
    for prob in (0.2, 0.5, 0.8):
        part = O.verify_step(hd, hd, W, K, block, 3, n_rm=3, recorrupt_prob=prob)
        assert np.all(part.remask <= full.remask)                      # only selected positions
        assert np.array_equal(part.tokens, full.tokens)                 # nothing else changes
        assert np.array_equal(part.conf, full.conf)
        assert part.pass_mask.sum() == 0                                # next pass starts with empty C
        for b in range(B):
            sel = np.flatnonzero(full.remask[b])
            u = philox.uniform(3, sel, 0, b, 3)
            assert np.array_equal(np.flatnonzero(part.remask[b]), sel[u < prob])
        total += int(part.remask.sum())
    assert 0 < total < 3 * 3 * B
    # a final pass re-corrupts nothing whatever the probability
    fin = O.verify_step(hd, hd, W, K, block, 3, n_rm=3, recorrupt_prob=0.5, final_pass=True)
    assert fin.remask.sum() == 0


def test_decode_passes_with_partial_recorruption():
    B, K, block = 4, 4, 12
    W, hidden = _laws(6, B, K, 32, 24)
    base = D.decode_block(hidden, W, B, K, block, seed=7, n_pass=3, n_rm=6)
    part = D.decode_block(hidden, W, B, K, block, seed=7, n_pass=3, n_rm=6, recorrupt_prob=0.4)
    assert np.all(part.X >= 0)
    for b in range(B):
        cp, rp = part.committed_per_pass[b], part.rounds_per_pass[b]
        assert cp[0] == block and rp[0] == base.rounds_per_pass[b][0]   # pass 0 is untouched
        for s in range(1, 3):
            assert cp[s] <= min(6, cp[s - 1])                           # at most the selection returns
            assert (cp[s] == 0) == (rp[s] == 0)                         # nothing masked: no round
        assert part.rounds[b] == sum(rp) <= base.rounds[b] + block
    assert sum(sum(c[1:]) for c in part.committed_per_pass) < sum(sum(c[1:]) for c in base.committed_per_pass)
    # probability one is the default behaviour, bit for bit
    one = D.decode_block(hidden, W, B, K, block, seed=7, n_pass=3, n_rm=6, recorrupt_prob=1.0)
    assert np.array_equal(one.X, base.X) and np.array_equal(one.rounds, base.rounds)


def test_tiny_probability_ends_the_decode_after_the_first_pass():
    B, K, block = 3, 4, 8
    W, hidden = _laws(8, B, K, 32, 24)
    first = D.decode_block(hidden, W, B, K, block, seed=2, n_pass=1)
    res = D.decode_block(hidden, W, B, K, block, seed=2, n_pass=4, n_rm=4, recorrupt_prob=5e-8)
    # the smallest uniform of the grid is 2^-24 = 5.96e-8 > 5e-8: nothing can be re-corrupted
    assert np.array_equal(res.X, first.X)
    for b in range(B):
        assert res.rounds_per_pass[b][1:] == [0, 0, 0]
