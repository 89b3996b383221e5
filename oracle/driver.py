"""Oracle for the outer loops of Algorithm 2 (full-sequence decoding) over one block.

TEST INFRASTRUCTURE (part of the CPU oracle; shares no code with the HIP path).

Algorithm 2, for one sequence:

    for s = 0 .. N_step-1:
        C^(s) <- {}
        while an unresolved position exists:      one speculative round (fef_oracle.verify_step)
        if s < N_step-1: R <- LowConf_{n_rm}(C^(s)); re-corrupt X^i for i in R

The model forwards are outside this build, so the hidden states of round r are given:
`hidden(r)` returns (h_draft, h_target) of shape [B, K, d] for the r-th round counted from the
start of the block; sequence b uses row b of round r for its own r-th round.  verify_step applies
LowConf inside the round that resolves the block, so the while-loop of pass s ends with that round
and the next pass starts from the re-masked positions.  Re-corrupted positions hold MASK (-1)
in X until they are committed again.

With recorrupt_prob < 1 a selected position returns to MASK only with that probability; a pass whose
selection re-corrupts nothing has no unresolved position, so its while-loop and those of all later
passes run zero rounds and X is final.

Pinned in tests: every position is committed exactly once per pass it belongs to, pass s >= 1
re-resolves exactly min(n_rm, candidates) positions (recorrupt_prob = 1), the number of rounds of a pass is at least
ceil(L / k), the final X has no MASK, and a run with N_step = 1 equals chaining verify_step by
hand.
"""
from dataclasses import dataclass

import numpy as np

from . import fef_oracle as O

MASK = -1


@dataclass
class DecodeResult:
    X: np.ndarray            # [B, block] final tokens of the block
    rounds: np.ndarray       # [B] speculative rounds used
    rounds_per_pass: list    # per sequence: rounds of each pass
    committed_per_pass: list  # per sequence: positions committed in each pass
    min_margin: np.ndarray   # [B] smallest decision margin met on the way (accept / CDF / LowConf)
    conf: np.ndarray         # [B, block] final confidences
    alpha_mean: np.ndarray   # [B] mean acceptance probability over the slots that were tested


def decode_block(hidden, W, B, K, block, seed, n_pass, n_rm=-1, temperature=1.0, seq_base=0,
                 pos_base=0, step_base=0, lowconf_scope=0, max_rounds=None, recorrupt_prob=1.0,
                 greedy=False):
    W = np.asarray(W, dtype=np.float64)
    X = np.full((B, block), MASK, np.int64)
    conf_out = np.zeros((B, block))
    rounds = np.zeros(B, np.int64)
    rpp, cpp = [], []
    min_margin = np.full(B, np.inf)
    alpha_mean = np.zeros(B)
    if max_rounds is None:
        max_rounds = block + n_pass * block
    for b in range(B):
        mask = np.ones((1, block), np.uint8)          # X <- X_t: the whole block is corrupted
        pmask = np.zeros((1, block), np.uint8)
        conf = np.zeros((1, block))
        r = 0
        rp, cp, alphas = [], [], []
        for s in range(n_pass):
            pmask[:] = 0                                # C^(s) <- {}
            n_rounds = n_commit = 0
            while mask.any():
                assert r < max_rounds
                hd, ht = hidden(r)
                res = O.verify_step(hd[b:b + 1], ht[b:b + 1], W, K, block, seed, temperature=temperature,
                                    step=step_base + r, seq_base=seq_base + b, pos_base=pos_base, n_rm=n_rm,
                                    final_pass=(s == n_pass - 1), lowconf_scope=lowconf_scope,
                                    mask_in=mask, pass_mask=pmask, conf=conf, recorrupt_prob=recorrupt_prob,
                                    greedy=greedy)
                C = int(res.committed[0])
                for m in range(C):
                    X[b, res.slot_pos[0, m]] = res.tokens[0, m]
                w = int(res.window[0])
                a = int(res.accept_len[0])
                last = min(a, w - 1)
                marg = min(res.accept_margin[0, :last + 1].min() / 10.0,   # accept tolerance is 10x the CDF one
                           res.draft_gap[0, :last + 1].min(),
                           res.resid_gap[0] if a < w else np.inf,
                           res.lowconf_gap[0],
                           np.inf if res.argmax_gap is None else res.argmax_gap[:, 0, :last + 1].min() / 100.0)
                min_margin[b] = min(min_margin[b], marg)
                alphas.extend(res.alpha[0, :last + 1].tolist())
                resolved = int(mask.sum()) - C == 0
                mask, pmask, conf = res.remask, res.pass_mask, res.conf
                r += 1; n_rounds += 1; n_commit += C
                if resolved:
                    X[b, mask[0] != 0] = MASK           # re-corrupted positions (none on the final pass)
                    break
            rp.append(n_rounds); cp.append(n_commit)
        rounds[b] = r
        rpp.append(rp); cpp.append(cp)
        conf_out[b] = conf[0]
        alpha_mean[b] = float(np.mean(alphas)) if alphas else 0.0
    return DecodeResult(X=X, rounds=rounds, rounds_per_pass=rpp, committed_per_pass=cpp,
                        min_margin=min_margin, conf=conf_out, alpha_mean=alpha_mean)
