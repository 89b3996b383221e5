"""Oracle for the training-side use of the vocabulary head: the token-level cross-entropy of
Algorithm 1 (position-conditioned training), forward only, plain numpy in fp64.

TEST INFRASTRUCTURE (part of the CPU oracle; shares no code with the HIP path).

For each prediction position j_m of a training sample, Algorithm 1 builds the position-conditioned
input X^(j_m), runs the predictor and takes

    CE_{j_m} = -log p_theta(X_0^{j_m} | X^(j_m), t),      L = sum_m CE_{j_m}.

The model forward is outside this build: row m of `h` is the predictor's hidden state at position
j_m for input X^(j_m), and p_theta = softmax(h_m W^T / tau) through the same bias-free vocabulary
head the decoding path uses (tau = 1 in training).  What is computed is therefore exactly the
definition: a log-softmax of the head's logits evaluated at the clean token.

Reading: a negative label marks a row that does not count (CE 0), so that a fixed-size batch of
rows can carry fewer than L_t positions.
"""
import numpy as np


def cross_entropy(h, W, labels, temperature=1.0):
    """h [R, d], W [V, d], labels [R] -> (ce [R], loss = sum of ce) in fp64."""
    h = np.asarray(h, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    labels = np.asarray(labels, dtype=np.int64)
    R, V = h.shape[0], W.shape[0]
    assert labels.shape == (R,) and np.all(labels < V)
    ce = np.zeros(R)
    for m in range(R):
        if labels[m] < 0:
            continue
        logits = (W @ h[m]) / temperature             # [V]
        top = logits.max()
        log_z = top + np.log(np.sum(np.exp(logits - top)))
        ce[m] = log_z - logits[labels[m]]
    return ce, float(ce.sum())
