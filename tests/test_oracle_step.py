"""Pins for the oracle's full speculative round (Algorithm 2) against what the paper proves:
the emitted token follows the target law (Theorem 1, one-step identity), the acceptance
probability is sum_v min(p_v, q_v), the committed length follows Theorem 2, plus special
cases, the window boundary and the LowConf re-corruption."""
import numpy as np
import pytest
import scipy.special
from scipy import stats

from oracle import fef_oracle as O
from oracle import philox


def _fixed_laws(V, d, K, seed, scale=2.0, rho=0.5):
    """One hidden-state pair per slot with logit std ~ scale, so the residual branch carries
    real mass (alpha roughly 0.5-0.7)."""
    rng = np.random.default_rng(seed)
    W = rng.normal(size=(V, d)) * 0.02
    s = scale / (0.02 * np.sqrt(d))
    hd = rng.normal(size=(K, d)) * s
    ht = rho * hd + np.sqrt(1 - rho ** 2) * rng.normal(size=(K, d)) * s
    q = scipy.special.softmax(hd @ W.T, axis=-1)
    p = scipy.special.softmax(ht @ W.T, axis=-1)
    return W, hd, ht, p, q


def _chi2_p(counts, probs):
    n = counts.sum()
    chi2 = np.sum((counts - n * probs) ** 2 / (n * probs))
    return stats.chi2.sf(chi2, len(probs) - 1)


def test_emitted_law_equals_target_brute_force_v8():
    """10^6 independent single-slot rounds on one fixed (p, q) at V=8: the committed token is
    distributed as p, the draft token as q, and the acceptance frequency is sum min(p, q)."""
    V, d, n = 8, 16, 1_000_000
    W, hd, ht, p, q = _fixed_laws(V, d, 1, seed=10)
    alpha = np.minimum(p[0], q[0]).sum()
    assert 0.3 < alpha < 0.9
    res = O.verify_step(np.broadcast_to(hd, (n, 1, d)), np.broadcast_to(ht, (n, 1, d)), W,
                        K=1, block=1, seed=1234)
    emitted = np.bincount(res.tokens[:, 0], minlength=V)
    drafted = np.bincount(res.draft_tokens[:, 0], minlength=V)
    assert _chi2_p(emitted, p[0]) > 1e-3
    assert _chi2_p(drafted, q[0]) > 1e-3
    # the emitted law must be distinguishable from the draft law at this sample size
    assert _chi2_p(emitted, q[0]) < 1e-6
    acc = (res.accept_len == 1).mean()
    assert abs(acc - alpha) < 4 * np.sqrt(alpha * (1 - alpha) / n)
    assert np.allclose(res.alpha[:, 0], alpha, atol=1e-12)
    # rejected rounds alone follow the residual law
    rej = res.accept_len == 0
    resid = np.maximum(p[0] - q[0], 0)
    resid /= resid.sum()
    keep = resid > 0
    counts = np.bincount(res.tokens[rej, 0], minlength=V)
    assert counts[~keep].sum() == 0
    assert _chi2_p(counts[keep], resid[keep]) > 1e-3


def test_second_slot_law_given_first_accepted():
    """Left-to-right verification: conditional on slot 1 being accepted, the token committed
    at slot 2 follows the target law of slot 2 (sequential step of Theorem 1's proof)."""
    V, d, n = 6, 16, 400_000
    W, hd, ht, p, q = _fixed_laws(V, d, 2, seed=11)
    res = O.verify_step(np.broadcast_to(hd, (n, 2, d)), np.broadcast_to(ht, (n, 2, d)), W,
                        K=2, block=2, seed=99)
    first_ok = res.accept_len >= 1
    assert np.all(res.tokens[~first_ok, 1] == -1)
    assert np.all(res.tokens[first_ok, 1] >= 0)
    counts = np.bincount(res.tokens[first_ok, 1], minlength=V)
    assert _chi2_p(counts, p[1]) > 1e-3
    # and the first slot, accepted or corrected, follows p of slot 1
    assert _chi2_p(np.bincount(res.tokens[:, 0], minlength=V), p[0]) > 1e-3


def test_mean_committed_length_matches_theorem_2():
    V, d, K, n = 8, 16, 8, 200_000
    W, hd, ht, p, q = _fixed_laws(V, d, K, seed=12, rho=0.8)
    alphas = np.minimum(p, q).sum(-1)
    res = O.verify_step(np.broadcast_to(hd, (n, K, d)), np.broadcast_to(ht, (n, K, d)), W,
                        K=K, block=K, seed=5)
    C = res.committed.astype(np.float64)
    want = O.expected_committed(alphas)
    assert abs(C.mean() - want) < 4 * C.std() / np.sqrt(n)
    assert np.all(res.committed == np.minimum(res.accept_len + 1, K))
    assert res.committed.max() <= K                       # no extra token after a full window
    # identical slots reduce to the closed form (1 - alpha^k)/(1 - alpha)
    hd1, ht1 = np.repeat(hd[:1], K, 0), np.repeat(ht[:1], K, 0)
    res1 = O.verify_step(np.broadcast_to(hd1, (n, K, d)), np.broadcast_to(ht1, (n, K, d)), W,
                         K=K, block=K, seed=6)
    C1 = res1.committed.astype(np.float64)
    assert abs(C1.mean() - O.expected_committed_iid(alphas[0], K)) < 4 * C1.std() / np.sqrt(n)


def test_theorem_2_closed_form():
    for a in [0.0, 0.3, 0.944, 0.999999]:
        for k in [1, 4, 16]:
            assert O.expected_committed_iid(a, k) == pytest.approx(sum(a ** l for l in range(k)), rel=1e-9)
            assert O.expected_committed([a] * k) == pytest.approx(sum(a ** l for l in range(k)), rel=1e-9)
    assert O.expected_committed_iid(1.0, 16) == 16
    assert O.acceleration_ratio(1.0, 16) == 8
    assert O.acceleration_ratio(0.5, 4, c_draft=1, c_target=3) == pytest.approx(1.875 * 0.75)


def test_identical_models_accept_everything():
    V, d, K = 32, 64, 4
    rng = np.random.default_rng(13)
    W = rng.normal(size=(V, d)) * 0.02
    h = rng.normal(size=(5, K, d)) * 20
    res = O.verify_step(h, h, W, K=K, block=8, seed=0)
    assert np.all(res.accept_len == K)
    assert np.array_equal(res.tokens, res.draft_tokens)
    assert np.all(res.resid_mass == 0) and np.allclose(res.alpha, 1)
    assert res.resid_fallbacks == 0
    assert np.all(res.committed == K)


def test_peaked_target_rejects_and_residual_is_target():
    V, d = 16, 16
    W = np.eye(V, d)
    hd = np.zeros((2000, 1, d)); hd[:, 0, 3] = 12.0        # draft law peaked on token 3
    ht = np.zeros((2000, 1, d)); ht[:, 0, 7] = 12.0        # target law peaked on token 7
    res = O.verify_step(hd, ht, W, K=1, block=1, seed=3)
    assert (res.accept_len == 0).mean() > 0.99
    assert (res.tokens[:, 0] == 7).mean() > 0.99
    assert np.all(res.resid_mass > 0.99)


def test_supplied_draft_tokens_ratio_direction_and_threshold():
    """K=1 with given draft tokens is textbook speculative sampling: a token with p >= q is
    always accepted, one with p < q is accepted with frequency p/q."""
    V, d, n = 8, 16, 100_000
    W, hd, ht, p, q = _fixed_laws(V, d, 1, seed=14)
    up = int(np.argmax(p[0] / q[0])); down = int(np.argmin(p[0] / q[0]))
    assert p[0, up] > q[0, up] and p[0, down] < q[0, down]
    H = np.broadcast_to(hd, (n, 1, d)); T = np.broadcast_to(ht, (n, 1, d))
    r_up = O.verify_step(H, T, W, K=1, block=1, seed=1, draft_tokens=np.full((n, 1), up))
    assert np.all(r_up.accept_len == 1) and np.all(r_up.tokens[:, 0] == up)
    r_dn = O.verify_step(H, T, W, K=1, block=1, seed=1, draft_tokens=np.full((n, 1), down))
    ratio = p[0, down] / q[0, down]
    f = (r_dn.accept_len == 1).mean()
    assert abs(f - ratio) < 4 * np.sqrt(ratio * (1 - ratio) / n)
    # the decision is exactly u <= ratio with the documented uniform
    u = philox.uniform(1, 0, 0, np.arange(n), philox.STREAM_ACCEPT)
    assert np.array_equal(r_dn.accept_len == 1, u <= ratio)
    assert np.allclose(r_dn.accept_margin[:, 0], np.abs(u - ratio))
    # confidences are the target probabilities of the committed tokens
    assert np.allclose(r_up.conf[:, 0], p[0, up])
    acc = r_dn.accept_len == 1
    assert np.allclose(r_dn.conf[acc, 0], p[0, down])
    assert np.allclose(r_dn.conf[~acc, 0], p[0, r_dn.tokens[~acc, 0]])


def test_temperature_scales_both_laws():
    V, d = 8, 16
    W, hd, ht, p, q = _fixed_laws(V, d, 1, seed=15)
    res = O.verify_step(hd[None], ht[None], W, K=1, block=1, seed=0, temperature=0.5,
                        return_logits=True)
    assert np.allclose(res.logits[0, 0, 0], 2 * hd[0] @ W.T)
    assert np.allclose(res.logits[1, 0, 0], 2 * ht[0] @ W.T)
    p2 = scipy.special.softmax(2 * ht[0] @ W.T); q2 = scipy.special.softmax(2 * hd[0] @ W.T)
    assert res.alpha[0, 0] == pytest.approx(np.minimum(p2, q2).sum())


def _small_batch(seed, B=6, K=4, d=32, V=32, block=8):
    rng = np.random.default_rng(seed)
    W = rng.normal(size=(V, d)) * 0.02
    s = 2.0 / (0.02 * np.sqrt(d))
    hd = rng.normal(size=(B, K, d)) * s
    ht = 0.7 * hd + np.sqrt(1 - 0.49) * rng.normal(size=(B, K, d)) * s
    return W, hd, ht


def test_output_conventions_and_window_boundary():
    W, hd, ht = _small_batch(20)
    mask = np.array([[1, 1, 1, 1, 1, 1, 1, 1],
                     [0, 0, 1, 0, 1, 0, 0, 1],      # three unresolved: window b = 3 < k
                     [0, 0, 0, 0, 0, 0, 1, 0],      # one unresolved
                     [0, 0, 0, 0, 0, 0, 0, 0],      # nothing to do
                     [1, 0, 1, 0, 1, 0, 1, 0],
                     [0, 1, 1, 1, 1, 1, 1, 1]], np.uint8)
    res = O.verify_step(hd, ht, W, K=4, block=8, seed=2, mask_in=mask, final_pass=True)
    assert res.window.tolist() == [4, 3, 1, 0, 4, 4]
    for b in range(6):
        a, w = res.accept_len[b], res.window[b]
        assert 0 <= a <= w
        C = min(a + 1, w)
        assert res.committed[b] == C
        assert np.all(res.tokens[b, :C] >= 0) and np.all(res.tokens[b, C:] == -1)
        assert np.array_equal(res.tokens[b, :a], res.draft_tokens[b, :a])
        cleared = np.flatnonzero(mask[b] & ~res.remask[b].astype(bool))
        assert cleared.tolist() == res.slot_pos[b, :C].tolist()       # exactly the committed slots
        assert np.array_equal(res.pass_mask[b], (mask[b] != 0) & (res.remask[b] == 0))
        assert np.all(res.remask[b] <= mask[b])                       # final pass: nothing re-masked
    assert res.accept_len[3] == 0 and res.committed[3] == 0


def test_uniforms_are_keyed_by_absolute_position_step_and_sequence():
    """Batch and shard invariance: a sequence's outcome depends only on its own rows and
    (seed, sequence id, step, position)."""
    W, hd, ht = _small_batch(21, B=5)
    full = O.verify_step(hd, ht, W, K=4, block=8, seed=9, step=3, seq_base=100, pos_base=64)
    for b in range(5):
        one = O.verify_step(hd[b:b + 1], ht[b:b + 1], W, K=4, block=8, seed=9, step=3,
                            seq_base=100 + b, pos_base=64)
        assert np.array_equal(one.tokens[0], full.tokens[b])
        assert one.accept_len[0] == full.accept_len[b]
        assert np.array_equal(one.remask[0], full.remask[b])
    again = O.verify_step(hd, ht, W, K=4, block=8, seed=9, step=3, seq_base=100, pos_base=64)
    assert np.array_equal(again.tokens, full.tokens)
    other_step = O.verify_step(hd, ht, W, K=4, block=8, seed=9, step=4, seq_base=100, pos_base=64)
    assert not np.array_equal(other_step.draft_tokens, full.draft_tokens)
    # the draft uniform of slot m is u(seed; pos_base + offset, step, seq, stream 0)
    q = scipy.special.softmax(hd[2, 1] @ W.T)
    u = philox.uniform(9, 64 + full.slot_pos[2, 1], 3, 102, philox.STREAM_DRAFT)
    assert full.draft_tokens[2, 1] == np.searchsorted(np.cumsum(q), u)
    # a shifted mask moves the position word and with it the draw
    mask = np.ones((5, 8), np.uint8); mask[:, 0] = 0
    shifted = O.verify_step(hd, ht, W, K=4, block=8, seed=9, step=3, seq_base=100, pos_base=63,
                            mask_in=mask)
    assert np.array_equal(shifted.draft_tokens, full.draft_tokens)


def _run_pass(W, hd_fn, K, block, seed, n_rm, final, scope=0, mask=None, conf=None, step0=0):
    """Drive rounds until the block is resolved once; returns the list of results."""
    B = 1
    mask = np.ones((B, block), np.uint8) if mask is None else mask
    pmask = np.zeros((B, block), np.uint8)
    conf = np.zeros((B, block)) if conf is None else conf
    out = []
    step = step0
    while True:
        hd, ht = hd_fn(step)
        before = mask.copy()
        res = O.verify_step(hd, ht, W, K=K, block=block, seed=seed, step=step, n_rm=n_rm,
                            final_pass=final, lowconf_scope=scope, mask_in=mask,
                            pass_mask=pmask, conf=conf)
        out.append((before, res))
        unresolved_after_commit = before[0].sum() - res.committed[0]
        mask, pmask, conf = res.remask, res.pass_mask, res.conf
        step += 1
        if unresolved_after_commit == 0:
            return out


def test_low_confidence_recorruption():
    V, d, K, block = 16, 16, 4, 8
    rng = np.random.default_rng(22)
    W = rng.normal(size=(V, d)) * 0.02
    s = 2.0 / (0.02 * np.sqrt(d))

    def hd_fn(step):
        r = np.random.default_rng(1000 + step)
        hd = r.normal(size=(1, K, d)) * s
        return hd, 0.8 * hd + 0.6 * r.normal(size=(1, K, d)) * s

    for n_rm in [0, 3, 4, 8, 20, -1]:
        rounds = _run_pass(W, hd_fn, K, block, seed=4, n_rm=n_rm, final=False)
        for before, res in rounds[:-1]:
            # block not yet resolved: nothing is re-masked, discarded drafts stay unresolved
            assert np.all(res.remask <= before)
            assert res.remask.sum() == before.sum() - res.committed[0]
        before, last = rounds[-1]
        want_n = min(block // 2 if n_rm < 0 else n_rm, block)     # whole block committed in this pass
        assert last.remask.sum() == want_n
        conf = last.conf[0]
        sel = np.flatnonzero(last.remask[0])
        rest = np.setdiff1d(np.arange(block), sel)
        order = sorted(range(block), key=lambda i: (conf[i], i))
        assert sorted(sel.tolist()) == sorted(order[:want_n])       # full-sort brute force
        if len(sel) and len(rest):
            assert conf[sel].max() <= conf[rest].min()
        assert last.pass_mask.sum() == 0                             # next pass starts with empty C
        # the same final round with final_pass set re-masks nothing
        fin = _run_pass(W, hd_fn, K, block, seed=4, n_rm=n_rm, final=True)[-1][1]
        assert fin.remask.sum() == 0
        assert np.array_equal(fin.tokens, last.tokens)


def test_low_confidence_scope():
    """Second pass over a block: the literal C^(s) holds only the positions re-resolved in
    this pass; scope 1 ranks every position of the block."""
    V, d, K, block = 16, 16, 2, 6
    rng = np.random.default_rng(23)
    W = rng.normal(size=(V, d)) * 0.02
    s = 2.0 / (0.02 * np.sqrt(d))

    def hd_fn(step):
        r = np.random.default_rng(2000 + step)
        hd = r.normal(size=(1, K, d)) * s
        return hd, 0.8 * hd + 0.6 * r.normal(size=(1, K, d)) * s

    mask = np.array([[0, 1, 0, 1, 1, 0]], np.uint8)        # three positions were re-masked
    conf0 = np.array([[1e-9, 0.5, 2e-9, 0.5, 0.5, 0.9]])    # old, very low confidences elsewhere
    lit = _run_pass(W, hd_fn, K, block, seed=8, n_rm=2, final=False, scope=0,
                    mask=mask.copy(), conf=conf0.copy(), step0=50)[-1][1]
    assert lit.remask.sum() == 2
    assert set(np.flatnonzero(lit.remask[0])) <= {1, 3, 4}
    alt = _run_pass(W, hd_fn, K, block, seed=8, n_rm=2, final=False, scope=1,
                    mask=mask.copy(), conf=conf0.copy(), step0=50)[-1][1]
    assert np.flatnonzero(alt.remask[0]).tolist() == [0, 2]
