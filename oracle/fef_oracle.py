"""Oracle for one FeF-DLLM speculative round (Algorithm 2, body of the while-loop, followed
by the low-confidence re-corruption of the same algorithm), plain numpy in fp64.

TEST INFRASTRUCTURE: only tests, the smoke check and the benchmark's cpu_baseline leg may
call this.  It shares no code with the HIP path.  Every function is pinned by the CPU test
suite against identities the paper proves (one-step identity in the proof of Theorem 1, the
residual-distribution equation, Theorem 2), library routines, brute force on tiny inputs and
the published Philox known-answer vectors.  Not pinned ("parity unpinned"): nothing that is
implemented here; classifier-free guidance is not implemented at all.

Notation follows the paper: rho / q = draft law, pi / p = target law, k = window, x~ = draft
token, C = committed positions, alpha = sum_v min(p_v, q_v).

The steps, in the paper's order (one call = one speculative round for B independent
sequences; all sequences are vectorised with numpy, the window is an explicit loop):

  S1  unresolved positions j_1 < ... < j_L of the block, window b = min(k, L)
      (Algorithm 2: "Let J_t ... be the unresolved positions", "Set b <- min{k, L_t}").
  S2  draft laws  rho^{j_m} = softmax(h_draft[m] W^T / tau)      ("Compute draft laws").
  S3  draft tokens x~^{j_m} ~ rho^{j_m} by inverse CDF           ("Sample draft tokens").
  S4  target laws pi^{j_m}  = softmax(h_target[m] W^T / tau)     ("Compute target laws").
      The model forwards that produce the hidden states are outside this step; the
      vocabulary head W is shared because draft and target are the same network
      (Experimental Setup).
  S5  left to right: u_m ~ U(0,1); accept iff u_m <= min{1, pi(x~)/rho(x~)};
      on acceptance commit x~ with confidence pi(x~);
      on the first rejection sample Z ~ pi' = [pi - rho]_+ / (1 - sum min{pi, rho})
      (residual-distribution equation), commit Z with confidence pi(Z), discard the rest.
  S6  when no unresolved position is left in the block and this is not the final pass:
      R = LowConf_{n_rm}(C^(s)) and every selected position is re-corrupted through the
      absorbing forward kernel q(X_t^i | X_0^i): MASK with probability recorrupt_prob
      (= 1 - alpha-bar_t of that kernel; 1 by default), otherwise it keeps its token.

  Greedy variant (greedy=True): the limit of S2-S5 as the sampling temperature goes to zero with
  the logits fixed.  Both laws become point masses at their arg max (lowest token id on a tie),
  so x~ = arg max of the draft logits, the ratio pi(x~)/rho(x~) is 1 when the two arg maxes agree
  and 0 otherwise (u > 0 always rejects), and the residual law is the target's point mass:
  Z = arg max of the target logits.  No uniform is drawn.  Confidences stay pi_tau(token) with
  the finite temperature given, the quantity LowConf ranks.

Readings of points the paper leaves open are listed with each function.
"""
from dataclasses import dataclass, field

import numpy as np

from . import philox


@dataclass
class StepResult:
    tokens: np.ndarray          # [B,K] int32: committed token per window slot, -1 = none
    accept_len: np.ndarray      # [B] int32: number of accepted drafts a (first rejection index)
    committed: np.ndarray       # [B] int32: C = min(a+1, b)  (Theorem 2's C_k)
    remask: np.ndarray          # [B,block] uint8: unresolved positions after the call
    pass_mask: np.ndarray       # [B,block] uint8: positions committed in the current pass
    conf: np.ndarray            # [B,block] float64: confidence pi(token) of resolved positions
    window: np.ndarray          # [B] int32: b = min(k, L)
    slot_pos: np.ndarray        # [B,K] int32: block offset of slot m, -1 if m >= b
    draft_tokens: np.ndarray    # [B,K] int32: x~, -1 if m >= b
    alpha: np.ndarray           # [B,K] float64: sum_v min(p_v, q_v)
    resid_mass: np.ndarray      # [B,K] float64: sum_v max(0, p_v - q_v)
    lse: np.ndarray             # [2,B,K] float64: log-sum-exp of (draft, target) logits
    p_draft_tok: np.ndarray     # [B,K] float64: pi(x~)
    q_draft_tok: np.ndarray     # [B,K] float64: rho(x~)
    accept_margin: np.ndarray   # [B,K] |u - min(1, pi/rho)|
    draft_gap: np.ndarray       # [B,K] distance of the draft uniform to the nearest CDF edge
    resid_gap: np.ndarray       # [B]   same for the residual draw, relative to the residual mass
    lowconf_gap: np.ndarray     # [B]   confidence gap at the LowConf selection boundary
    argmax_gap: np.ndarray = None  # [2,B,K] greedy only: top-1 minus top-2 scaled logit (draft, target)
    resid_fallbacks: int = 0    # times a rejection met a non-positive residual mass
    logits: np.ndarray = field(default=None, repr=False)  # [2,B,K,V] if requested


def head_logits(h, W, temperature):
    """Vocabulary-head projection L[..., v] = sum_k h[..., k] W[v, k] / tau.

    The hidden state is the input of a bias-free linear head shared by both laws.  Reading
    for the temperature (its value is only said to equal the baseline's): both laws are
    softmax(logits / tau), tau > 0.
    """
    return np.matmul(h, W.T) / temperature


def log_sum_exp(L):
    """log sum_v exp(L[..., v]), shifted by the row maximum."""
    mx = np.max(L, axis=-1, keepdims=True)
    return (mx + np.log(np.sum(np.exp(L - mx), axis=-1, keepdims=True)))[..., 0]


def law(L):
    """Categorical law softmax(L) along the last axis and its log-sum-exp."""
    lse = log_sum_exp(L)
    return np.exp(L - lse[..., None]), lse


def inverse_cdf(mass, target):
    """First index v (ascending token id) whose inclusive prefix sum reaches the target:
    min{v : sum_{w<=v} mass_w >= target}, per row.

    mass [B,V] non-negative, target [B].  If rounding leaves every prefix sum below the
    target, the last index with positive mass is returned.  Also returns the distance from
    the target to the nearer edge of the selected interval (+inf towards an edge that cannot
    be crossed: below token 0 and above the last token).
    """
    cdf = np.cumsum(mass, axis=-1)
    reached = cdf >= target[:, None]
    idx = np.argmax(reached, axis=-1)
    none = ~reached[:, -1]
    if np.any(none):
        V = mass.shape[-1]
        last_pos = V - 1 - np.argmax(mass[:, ::-1] > 0, axis=-1)
        idx = np.where(none, last_pos, idx)
    rows = np.arange(mass.shape[0])
    upper = cdf[rows, idx] - target
    lower = target - np.where(idx > 0, cdf[rows, np.maximum(idx - 1, 0)], -np.inf)
    upper = np.where(idx == mass.shape[-1] - 1, np.inf, upper)
    gap = np.minimum(np.abs(upper), np.abs(lower))
    return idx.astype(np.int64), gap


def residual_law(p, q):
    """Unnormalised residual [p - q]_+ and its mass, which the residual-distribution
    equation writes as 1 - sum_z min{p_z, q_z}."""
    r = np.maximum(p - q, 0.0)
    return r, np.sum(r, axis=-1)


def window_slots(mask, K):
    """Window of a block: slot m is the (m+1)-th unresolved position in ascending order,
    b = min(k, L).  Returns slot positions [B,K] (-1 beyond b) and b [B]."""
    B, block = mask.shape
    slot_pos = np.full((B, K), -1, dtype=np.int32)
    window = np.zeros(B, dtype=np.int32)
    for b in range(B):
        unresolved = np.flatnonzero(mask[b])
        n = min(K, unresolved.size)
        slot_pos[b, :n] = unresolved[:n]
        window[b] = n
    return slot_pos, window


def low_confidence(conf_row, candidates, n_rm):
    """LowConf_{n_rm}: the n_rm candidate positions with the smallest confidence; equal
    confidences are ordered by position.  Returns the selected positions and the confidence
    gap between the last selected and the first unselected candidate (+inf if every
    candidate is selected or none is)."""
    cand = np.flatnonzero(candidates)
    n = min(int(n_rm), cand.size)
    if n <= 0 or cand.size == 0:
        return cand[:0], np.inf
    order = cand[np.lexsort((cand, conf_row[cand]))]
    gap = np.inf
    if n < cand.size:
        gap = float(conf_row[order[n]] - conf_row[order[n - 1]])
    return order[:n], gap


def recorrupt(selected, prob, seed, pos_base, step, sequence):
    """Algorithm 2, "Re-corrupt X^i ~ q(X_t^i | X_0^i)" with the absorbing (mask) forward
    kernel of D3PM: position i becomes MASK with probability prob = 1 - alpha-bar_t and keeps
    its clean token otherwise, independently over positions.  Returns the positions that
    become MASK.

    Readings: the paper gives neither t nor the uniforms.  prob is an input (a binary32 number,
    as the boundary carries it; 1 reproduces "selected positions always return to MASK"); the
    draw for position i is Philox stream 3 at (absolute position, step, sequence) and the
    position is masked iff u < prob, both exact in binary32 and binary64."""
    selected = np.asarray(selected, dtype=np.int64)
    p = float(np.float32(prob))
    if p >= 1.0 or selected.size == 0:
        return selected
    u = philox.uniform(seed, pos_base + selected, step, sequence, philox.STREAM_RECORRUPT)
    return selected[u < p]


def verify_step(h_draft, h_target, W, K, block, seed, *, temperature=1.0, step=0,
                seq_base=0, pos_base=0, n_rm=-1, final_pass=False, lowconf_scope=0,
                mask_in=None, pass_mask=None, conf=None, draft_tokens=None,
                return_logits=False, recorrupt_prob=1.0, greedy=False, W_draft=None):
    """One speculative round for B sequences.

    h_draft, h_target: [B,K,d] float64 (row m belongs to window slot m); W: [V,d] float64.
    mask_in: [B,block] 1 = unresolved (None = whole block unresolved).
    pass_mask / conf: state of the current pass C^(s) (None = empty / zeros).
    draft_tokens: optional [B,K] tokens to verify instead of sampling them here.

    Readings where the paper is silent:
      * uniforms: Philox4x32-10 keyed (seed; absolute position, step, sequence, stream); the
        residual draw uses the position of the rejected slot.
      * accept test uses "<=" exactly as printed in Algorithm 2.
      * accept_len counts accepted drafts; the committed count is min(a+1, b): the corrected
        position is committed too and there is no extra token after a fully accepted window
        (Theorem 2: C_k <= k).
      * re-corruption is the absorbing kernel: a selected position becomes MASK with
        probability recorrupt_prob (see recorrupt()).  n_rm < 0 means block // 2.
      * LowConf ranges over the positions committed in the current pass (lowconf_scope 0,
        the literal C^(s)) or over every position of the resolved block (scope 1).
      * a rejection that meets residual mass <= 0 (cannot happen in exact arithmetic)
        commits argmax p and is counted in resid_fallbacks.
      * greedy=True: the zero-temperature limit described in the module header; `temperature`
        then only scales the logits the confidences are taken from.
      * W_draft: output embedding of a separate draft model ("A / B" of the ablation on the choice
        of draft model, Ablation 3 and Table 4): the draft laws are softmax(h_draft W_draft^T / tau), the target
        laws keep W.  None = one model for both, the paper's default.
    """
    h_draft = np.asarray(h_draft, dtype=np.float64)
    h_target = np.asarray(h_target, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    W_q = W if W_draft is None else np.asarray(W_draft, dtype=np.float64)
    assert W_q.shape == W.shape
    B, Kh, d = h_draft.shape
    V = W.shape[0]
    assert Kh == K and h_target.shape == h_draft.shape and W.shape[1] == d
    assert 1 <= K <= block and temperature > 0
    mask = np.ones((B, block), np.uint8) if mask_in is None else (np.asarray(mask_in) != 0).astype(np.uint8)
    pmask = np.zeros((B, block), np.uint8) if pass_mask is None else (np.asarray(pass_mask) != 0).astype(np.uint8)
    cf = np.zeros((B, block), np.float64) if conf is None else np.array(conf, dtype=np.float64)
    if n_rm < 0:
        n_rm = block // 2

    # S1: window
    slot_pos, window = window_slots(mask, K)
    seq = seq_base + np.arange(B)
    abs_pos = pos_base + np.maximum(slot_pos, 0)

    x_draft = np.full((B, K), -1, np.int64)
    alpha = np.zeros((B, K)); resid_mass = np.zeros((B, K))
    lse = np.zeros((2, B, K))
    p_tok = np.zeros((B, K)); q_tok = np.zeros((B, K))
    accept = np.zeros((B, K), bool)
    accept_margin = np.full((B, K), np.inf); draft_gap = np.full((B, K), np.inf)
    resid_tok = np.full((B, K), -1, np.int64); resid_conf = np.zeros((B, K))
    resid_gap_slot = np.full((B, K), np.inf)
    fallbacks = np.zeros((B, K), bool)
    logits = np.zeros((2, B, K, V)) if return_logits else None
    argmax_gap = np.full((2, B, K), np.inf) if greedy else None

    for m in range(K):
        active = m < window
        # S2 / S4: the two laws of slot m
        Lq = head_logits(h_draft[:, m, :], W_q, temperature)
        Lp = head_logits(h_target[:, m, :], W, temperature)
        q, lse_q = law(Lq)
        p, lse_p = law(Lp)
        lse[0, :, m], lse[1, :, m] = lse_q, lse_p
        if return_logits:
            logits[0, :, m], logits[1, :, m] = Lq, Lp
        alpha[:, m] = np.sum(np.minimum(p, q), axis=-1)
        r, resid_mass[:, m] = residual_law(p, q)

        if greedy and V > 1:
            for side, L in enumerate((Lq, Lp)):
                top2 = np.partition(L, V - 2, axis=-1)[:, V - 2:]
                argmax_gap[side, :, m] = top2[:, 1] - top2[:, 0]

        # S3: draft token
        if draft_tokens is None and greedy:
            x = np.argmax(Lq, axis=-1)            # point mass of the draft law; first index on a tie
        elif draft_tokens is None:
            u0 = philox.uniform(seed, abs_pos[:, m], step, seq, philox.STREAM_DRAFT)
            x, draft_gap[:, m] = inverse_cdf(q, u0)
        else:
            x = np.asarray(draft_tokens)[:, m].astype(np.int64)
            x = np.where(active, x, 0)
        rows = np.arange(B)
        x_draft[:, m] = np.where(active, x, -1)

        # S5: accept test  u <= min{1, pi(x~)/rho(x~)}
        u1 = philox.uniform(seed, abs_pos[:, m], step, seq, philox.STREAM_ACCEPT)
        log_ratio = (Lp[rows, x] - lse_p) - (Lq[rows, x] - lse_q)
        with np.errstate(over="ignore"):
            ratio = np.minimum(1.0, np.exp(log_ratio))
        accept[:, m] = u1 <= ratio
        accept_margin[:, m] = np.abs(u1 - ratio)
        p_tok[:, m], q_tok[:, m] = p[rows, x], q[rows, x]
        if greedy:                                  # ratio of the two point masses: 1 or 0
            accept[:, m] = x == np.argmax(Lp, axis=-1)
            accept_margin[:, m] = np.inf

        # residual sample for this slot (used only where slot m is the first rejection)
        u2 = philox.uniform(seed, abs_pos[:, m], step, seq, philox.STREAM_RESIDUAL)
        z, g = inverse_cdf(r, u2 * resid_mass[:, m])
        degenerate = resid_mass[:, m] <= 0.0
        z = np.where(degenerate, np.argmax(p, axis=-1), z)
        fallbacks[:, m] = degenerate
        if greedy:                                  # residual of two point masses = the target's
            z = np.argmax(Lp, axis=-1)
            g = np.full(B, np.inf)
            fallbacks[:, m] = False
            degenerate = np.zeros(B, bool)
        resid_tok[:, m] = z
        resid_conf[:, m] = p[rows, z]
        with np.errstate(divide="ignore", invalid="ignore"):
            resid_gap_slot[:, m] = np.where(degenerate, 0.0, g / resid_mass[:, m])

    # S5 (control flow): first rejection, commits and confidences
    tokens = np.full((B, K), -1, np.int32)
    accept_len = np.zeros(B, np.int32)
    committed = np.zeros(B, np.int32)
    resid_gap = np.full(B, np.inf)
    n_fallback = 0
    new_mask = mask.copy()
    for b in range(B):
        a = int(window[b])
        for m in range(int(window[b])):
            if accept[b, m]:
                tokens[b, m] = x_draft[b, m]
                cf[b, slot_pos[b, m]] = p_tok[b, m]
            else:
                a = m
                tokens[b, m] = resid_tok[b, m]
                cf[b, slot_pos[b, m]] = resid_conf[b, m]
                resid_gap[b] = resid_gap_slot[b, m]
                n_fallback += int(fallbacks[b, m])
            new_mask[b, slot_pos[b, m]] = 0
            pmask[b, slot_pos[b, m]] = 1
            if not accept[b, m]:
                break
        accept_len[b] = a
        committed[b] = min(a + 1, int(window[b]))

    # S6: low-confidence re-corruption once the block is resolved
    lowconf_gap = np.full(B, np.inf)
    final = np.broadcast_to(np.asarray(final_pass, dtype=bool), (B,))   # scalar or one flag per sequence
    for b in range(B):
        if not final[b]:
            if new_mask[b].any():
                continue
            cand = pmask[b] if lowconf_scope == 0 else np.ones(block, np.uint8)
            sel, lowconf_gap[b] = low_confidence(cf[b], cand, n_rm)
            new_mask[b, recorrupt(sel, recorrupt_prob, seed, pos_base, step, seq_base + b)] = 1
            pmask[b, :] = 0

    return StepResult(tokens=tokens, accept_len=accept_len, committed=committed,
                      remask=new_mask, pass_mask=pmask, conf=cf, window=window,
                      slot_pos=slot_pos, draft_tokens=x_draft.astype(np.int32), alpha=alpha,
                      resid_mass=resid_mass, lse=lse, p_draft_tok=p_tok, q_draft_tok=q_tok,
                      accept_margin=accept_margin, draft_gap=draft_gap, resid_gap=resid_gap,
                      lowconf_gap=lowconf_gap, resid_fallbacks=n_fallback, logits=logits,
                      argmax_gap=argmax_gap)


def expected_committed(alphas):
    """Theorem 2 for per-slot acceptance probabilities alpha_1..alpha_k with independent
    tests: E[C_k] = sum_{l=0}^{k-1} prod_{m<=l} alpha_m, which is sum_l alpha^l when all
    slots share one alpha."""
    alphas = np.asarray(alphas, dtype=np.float64)
    return float(np.sum(np.concatenate([[1.0], np.cumprod(alphas[:-1])])))


def expected_committed_iid(alpha, k):
    """Closed form of Theorem 2: (1 - alpha^k)/(1 - alpha), k at alpha = 1."""
    if alpha == 1.0:
        return float(k)
    return (1.0 - alpha ** k) / (1.0 - alpha)


def acceleration_ratio(alpha, k, c_draft=1.0, c_target=1.0):
    """Corollary 2: S = E[C_k] c_pi / (c_rho + c_pi)."""
    return expected_committed_iid(alpha, k) * c_target / (c_draft + c_target)
