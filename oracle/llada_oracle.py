"""Oracle for the baseline decoding step the paper measures its speed-ups against: LLaDA's
parallel prediction with top-n confidence transfer (n = 1: LLaDA, n = 2: the LLaDA/2 variant of
the Main Results), plain numpy in fp64.

TEST INFRASTRUCTURE (part of the CPU oracle; shares no code with the HIP path).

One step, per sequence, on the window of the first K unresolved positions of the block
(all of them when K >= their number):

  T1  law of every window position from ONE forward: p^{j_m} = softmax(h[m] W^T / tau)
      (the independent clean-token prediction the paper's Eq. for the standard X_0 predictor uses).
  T2  x^{j_m} ~ p^{j_m} by inverse CDF (ascending token id), or arg max when greedy.
  T3  confidence c_{j_m} = p^{j_m}(x^{j_m}).
  T4  the n positions with the highest confidence are committed (equal confidences: the lower
      position first); the others stay MASK.

The paper describes the baseline only as "decodes one token at each step" / "two tokens per step";
T2-T4 are the low-confidence re-masking rule of the LLaDA decoder it refers to, restated.  Uniforms
are the Philox draws of the speculative step's draft stream (stream 0) at the same counters.
"""
from dataclasses import dataclass

import numpy as np

from . import fef_oracle as O
from . import philox


@dataclass
class TopNResult:
    tokens: np.ndarray        # [B,K] int32: committed token per window slot, -1 = not committed
    committed: np.ndarray     # [B] int32: min(n, window)
    remask: np.ndarray        # [B,block] uint8: unresolved positions after the step
    conf: np.ndarray          # [B,block] float64: confidences (updated at committed positions)
    window: np.ndarray        # [B]
    slot_pos: np.ndarray      # [B,K]
    drawn: np.ndarray         # [B,K] int32: x of every window slot, -1 beyond the window
    slot_conf: np.ndarray     # [B,K] c of every window slot
    lse: np.ndarray           # [B,K]
    draw_gap: np.ndarray      # [B,K] distance of the uniform to the nearest CDF edge / arg max gap
    select_gap: np.ndarray    # [B] confidence gap at the selection boundary (+inf if none)


def topn_step(h, W, K, block, seed, n_transfer, *, temperature=1.0, step=0, seq_base=0, pos_base=0,
              mask_in=None, conf=None, greedy=False):
    h = np.asarray(h, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    B, Kh, d = h.shape
    V = W.shape[0]
    assert Kh == K and 1 <= K <= block and n_transfer >= 1 and temperature > 0
    mask = np.ones((B, block), np.uint8) if mask_in is None else (np.asarray(mask_in) != 0).astype(np.uint8)
    cf = np.zeros((B, block)) if conf is None else np.array(conf, dtype=np.float64)
    slot_pos, window = O.window_slots(mask, K)
    seq = seq_base + np.arange(B)
    abs_pos = pos_base + np.maximum(slot_pos, 0)
    drawn = np.full((B, K), -1, np.int64)
    slot_conf = np.zeros((B, K)); lse = np.zeros((B, K)); gap = np.full((B, K), np.inf)
    rows = np.arange(B)
    for m in range(K):
        L = O.head_logits(h[:, m, :], W, temperature)                # T1
        p, lse[:, m] = O.law(L)
        if greedy:                                                    # T2
            x = np.argmax(L, axis=-1)
            if V > 1:
                top2 = np.partition(L, V - 2, axis=-1)[:, V - 2:]
                gap[:, m] = top2[:, 1] - top2[:, 0]
        else:
            u = philox.uniform(seed, abs_pos[:, m], step, seq, philox.STREAM_DRAFT)
            x, gap[:, m] = O.inverse_cdf(p, u)
        active = m < window
        drawn[:, m] = np.where(active, x, -1)
        slot_conf[:, m] = np.where(active, p[rows, x], 0.0)          # T3
    tokens = np.full((B, K), -1, np.int32)
    committed = np.zeros(B, np.int32)
    new_mask = mask.copy()
    select_gap = np.full(B, np.inf)
    for b in range(B):                                                # T4
        w = int(window[b])
        order = sorted(range(w), key=lambda m: (-slot_conf[b, m], slot_pos[b, m]))
        n = min(int(n_transfer), w)
        for m in order[:n]:
            tokens[b, m] = drawn[b, m]
            new_mask[b, slot_pos[b, m]] = 0
            cf[b, slot_pos[b, m]] = slot_conf[b, m]
        committed[b] = n
        if 0 < n < w:
            select_gap[b] = slot_conf[b, order[n - 1]] - slot_conf[b, order[n]]
    return TopNResult(tokens=tokens, committed=committed, remask=new_mask, conf=cf, window=window,
                      slot_pos=slot_pos, drawn=drawn.astype(np.int32), slot_conf=slot_conf, lse=lse,
                      draw_gap=gap, select_gap=select_gap)
