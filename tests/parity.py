"""Comparison of a HIP verify step with the CPU oracle on the same inputs.

Discrete outputs (tokens, accepted length, re-mask set) must be bit-exact.  The one exception
is a decision that floating point cannot separate: the oracle reports, per slot, how far each
uniform was from the boundary it was compared with.  A sequence whose outcome hinges on a
boundary closer than the tolerances below is counted as near-margin; it is still compared, and
only there may the two sides differ (a flipped decision changes everything after it) - such
flips are counted separately.  Tolerances:

  accept test     |u - min(1, p/q)| < 1e-4     (fp32 log-ratio of four logits/lse terms)
  inverse CDFs    gap to the nearest CDF edge < 1e-5 (relative to the residual mass for the
                  residual draw): fp32 prefix sums over up to 1.5e5 probabilities whose logits
                  carry ~1e-5 absolute error from fp32 accumulation over d = 4096
  LowConf         confidence gap at the selection boundary < 1e-5

Continuous outputs: logits and probabilities within 2e-2 relative (the stated bound) and
within the much tighter bounds derived from fp32 accumulation; overlap / residual masses
within 1e-5 absolute.
"""
import numpy as np

TOL_ACCEPT = 1e-4
TOL_CDF = 1e-5
TOL_CONF = 1e-5
TOL_MASS = 1e-5
TOL_ARGMAX = 1e-3     # greedy variant: top-1 minus top-2 scaled logit (5 x the logit tolerance)


def compare(ref, tokens, accept_len, remask, diag=None, drafts_given=False, logit_atol=2e-4):
    """ref: oracle StepResult; tokens/accept_len/remask: numpy arrays from the HIP path;
    diag: dict of numpy arrays (optional).  Returns counters; raises AssertionError on mismatch."""
    B, K = ref.tokens.shape
    stats = {"sequences": B, "equal": 0, "near_margin": 0, "near_flipped": 0, "compared": 0,
             "remask_skipped": 0, "draft_slots": 0, "draft_near": 0}
    for b in range(B):
        w, a = int(ref.window[b]), int(ref.accept_len[b])
        last = min(a, w - 1)
        near = False
        for m in range(last + 1):
            if not drafts_given and ref.draft_gap[b, m] < TOL_CDF:
                near = True
            if ref.accept_margin[b, m] < TOL_ACCEPT:
                near = True
        if a < w and ref.resid_gap[b] < TOL_CDF:
            near = True
        if ref.argmax_gap is not None and w > 0 and ref.argmax_gap[:, b, :last + 1].min() < TOL_ARGMAX:
            near = True
        near_remask = ref.lowconf_gap[b] < TOL_CONF
        same = int(accept_len[b]) == a and np.array_equal(tokens[b], ref.tokens[b])
        same_remask = np.array_equal(remask[b], ref.remask[b])
        stats["near_margin"] += int(near)
        stats["compared"] += int(not near)
        if same and (same_remask or near_remask):
            stats["equal"] += 1
            stats["remask_skipped"] += int(not same_remask)
            continue
        # a difference is tolerated only where the oracle says the decision was within rounding
        assert near, (f"seq {b}: accept_len {accept_len[b]} vs {a}, tokens {tokens[b]} vs {ref.tokens[b]}, "
                      f"remask {remask[b]} vs {ref.remask[b]}")
        stats["near_flipped"] += 1
    if diag is not None:
        active = np.arange(K)[None, :] < ref.window[:, None]
        if "draft_tokens" in diag and not drafts_given:
            ok = active & (ref.draft_gap >= TOL_CDF)
            if ref.argmax_gap is not None:
                ok &= ref.argmax_gap[0] >= TOL_ARGMAX
            stats["draft_slots"] = int(active.sum())
            stats["draft_near"] = int((active & ~ok).sum())
            assert np.array_equal(diag["draft_tokens"][ok], ref.draft_tokens[ok])
            assert np.all(diag["draft_tokens"][~active] == -1)
        if "lse" in diag:
            d = np.abs(diag["lse"] - ref.lse)
            assert np.all(d <= 2e-2 * np.abs(ref.lse) + 1e-6)
            assert d.max() <= 1e-4, f"lse error {d.max()}"
            stats["lse_err"] = float(d.max())
        if "alpha" in diag:
            d = np.abs(diag["alpha"] - ref.alpha)[active]
            assert d.size == 0 or d.max() <= TOL_MASS, f"alpha error {d.max()}"
            stats["alpha_err"] = float(d.max()) if d.size else 0.0
        if "resid_mass" in diag:
            d = np.abs(diag["resid_mass"] - ref.resid_mass)[active]
            assert d.size == 0 or d.max() <= TOL_MASS, f"residual mass error {d.max()}"
            stats["resid_err"] = float(d.max()) if d.size else 0.0
        if "logits" in diag and ref.logits is not None:
            d = np.abs(diag["logits"] - ref.logits)
            assert np.all(d <= 2e-2 * np.abs(ref.logits) + logit_atol)
            assert d.max() <= logit_atol, f"logit error {d.max()}"
            stats["logit_err"] = float(d.max())
        if "conf_tok" in diag:
            # confidences of the committed tokens, where the committed token is the oracle's
            same = (tokens == ref.tokens) & (ref.tokens >= 0)
            want = np.zeros((B, K))
            for b in range(B):
                for m in range(K):
                    if ref.tokens[b, m] >= 0:
                        want[b, m] = ref.conf[b, ref.slot_pos[b, m]]
            got = diag["conf_tok"]
            rel = np.abs(got - want)[same] / np.maximum(want[same], 1e-30)
            assert rel.size == 0 or rel.max() <= 2e-2
            assert rel.size == 0 or rel.max() <= 2e-4, f"confidence rel error {rel.max()}"
            stats["conf_rel_err"] = float(rel.max()) if rel.size else 0.0
    return stats
