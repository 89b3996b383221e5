"""GPU parity of the device-side Algorithm 2 loop state (pass counters, token state, LowConf at
block resolution) against the oracle's outer loops, with rounds queued back to back and nothing
read back in between."""
import numpy as np
import pytest
import torch

from oracle import driver as D
from oracle import fef_oracle as O
from paper_2605_14305_amd import binding as fb
from paper_2605_14305_amd import synth
import parity

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _run(B, K, block, d, V, n_pass, n_rm, seed, rho=0.85, variant=fb.FEF_GEMM_AUTO, scope=0, recorrupt_prob=1.0,
         greedy=False):
    W = synth.make_head(V, d, seed)
    sigma = 3.0 / (0.02 * np.sqrt(d))
    vs = fb.VerifyStep(B, K, block, d, V, device=DEV, gemm_variant=variant)
    dec = fb.BlockDecoder(vs, n_pass, n_rm, scope, recorrupt_prob, greedy)
    R = dec.max_rounds()
    rounds = [synth.make_hidden(B, K, d, seed, rho, sigma, "bf16", 3, r) for r in range(R)]
    Wd = W.to(DEV)
    dev_rounds = [(hd.to(DEV), ht.to(DEV)) for hd, ht in rounds]
    torch.cuda.synchronize()
    for r in range(R):                       # no synchronisation inside the loop
        dec.round(dev_rounds[r][0], dev_rounds[r][1], Wd, seed, step=100 + r, pos_base=96, seq_base=20)
    torch.cuda.synchronize()
    f64 = {}

    def hidden(r):
        if r not in f64:
            f64[r] = (synth.to_f64(rounds[r][0]), synth.to_f64(rounds[r][1]))
        return f64[r]
    ref = D.decode_block(hidden, synth.to_f64(W), B, K, block, seed, n_pass, n_rm, seq_base=20, pos_base=96,
                         step_base=100, lowconf_scope=scope, max_rounds=R, recorrupt_prob=recorrupt_prob,
                         greedy=greedy)
    return dec, ref


@pytest.mark.parametrize("n_pass,n_rm,scope,variant", [(1, -1, 0, fb.FEF_GEMM_AUTO), (3, 5, 0, fb.FEF_GEMM_AUTO),
                                                       (2, -1, 1, fb.FEF_GEMM_SKINNY), (4, 3, 0, fb.FEF_GEMM_TILED)])
def test_block_decode_matches_algorithm_2(n_pass, n_rm, scope, variant):
    B, K, block, d, V = (1 if variant == fb.FEF_GEMM_SKINNY else 6), 4, 16, 512, 900
    dec, ref = _run(B, K, block, d, V, n_pass, n_rm, seed=31 + n_pass, variant=variant, scope=scope)
    X, rounds, sp = dec.tokens.cpu().numpy(), dec.seq_rounds.cpu().numpy(), dec.seq_pass.cpu().numpy()
    assert np.all(dec.mask.cpu().numpy() == 0)            # every sequence finished within max_rounds
    assert np.all(sp == n_pass)                           # ... and says so
    assert np.all(X >= 0)
    equal = 0
    for b in range(B):
        same = np.array_equal(X[b], ref.X[b]) and rounds[b] == ref.rounds[b]
        equal += int(same)
        if ref.min_margin[b] < parity.TOL_CDF:            # some decision on the way was within rounding:
            continue                                      # a difference is tolerated, and counted
        assert same, (b, X[b], ref.X[b], rounds[b], ref.rounds[b])
        assert np.allclose(dec.conf.cpu().numpy()[b], ref.conf[b], rtol=2e-4, atol=1e-12)
    print(f"n_pass={n_pass}: {equal}/{B} sequences identical to the oracle, "
          f"{int((ref.min_margin < parity.TOL_CDF).sum())} had a near-margin decision", flush=True)
    assert equal >= B - 1


@pytest.mark.parametrize("prob", [0.5, 0.15])
def test_block_decode_with_stochastic_recorruption(prob):
    """Passes whose LowConf selection is re-corrupted with probability < 1, including sequences
    where a selection re-corrupts nothing and the remaining passes are empty."""
    B, K, block, d, V, n_pass = 8, 4, 16, 512, 900, 4
    dec, ref = _run(B, K, block, d, V, n_pass, 3, seed=77, recorrupt_prob=prob)
    X, rounds, sp = dec.tokens.cpu().numpy(), dec.seq_rounds.cpu().numpy(), dec.seq_pass.cpu().numpy()
    assert np.all(dec.mask.cpu().numpy() == 0) and np.all(sp == n_pass) and np.all(X >= 0)
    equal = 0
    for b in range(B):
        same = np.array_equal(X[b], ref.X[b]) and rounds[b] == ref.rounds[b]
        equal += int(same)
        if ref.min_margin[b] < parity.TOL_CDF:
            continue
        assert same, (b, X[b], ref.X[b], rounds[b], ref.rounds[b])
        assert np.allclose(dec.conf.cpu().numpy()[b], ref.conf[b], rtol=2e-4, atol=1e-12)
    redo = [sum(c[1:]) for c in ref.committed_per_pass]
    print(f"prob={prob}: {equal}/{B} identical, re-resolved positions per sequence {redo}", flush=True)
    assert equal >= B - 1
    assert min(redo) < 3 * (n_pass - 1)                    # some selection was only partly re-corrupted


def test_block_decode_greedy():
    """Greedy rounds queued back to back over two passes: tokens, round counts and confidences."""
    B, K, block, d, V, n_pass = 6, 4, 16, 512, 900, 2
    dec, ref = _run(B, K, block, d, V, n_pass, 4, seed=88, rho=0.93, greedy=True)
    X, rounds, sp = dec.tokens.cpu().numpy(), dec.seq_rounds.cpu().numpy(), dec.seq_pass.cpu().numpy()
    assert np.all(dec.mask.cpu().numpy() == 0) and np.all(sp == n_pass) and np.all(X >= 0)
    equal = 0
    for b in range(B):
        same = np.array_equal(X[b], ref.X[b]) and rounds[b] == ref.rounds[b]
        equal += int(same)
        if ref.min_margin[b] < parity.TOL_CDF:
            continue
        assert same, (b, X[b], ref.X[b], rounds[b], ref.rounds[b])
        assert np.allclose(dec.conf.cpu().numpy()[b], ref.conf[b], rtol=2e-4, atol=1e-12)
    print(f"greedy: {equal}/{B} identical, rounds {rounds.tolist()}", flush=True)
    assert equal >= B - 1


def test_block_decode_llada_shape_rounds_vs_expected_length():
    """LLaDA-shaped block (d=4096, V=126464, block 32, K=8, two passes): final tokens equal the
    oracle's; reports rounds per block against block / E[C_k]."""
    wl = synth.WORKLOADS["llada_b1"]
    dec, ref = _run(1, wl.K, wl.block, wl.d, wl.V, n_pass=2, n_rm=-1, seed=4, rho=wl.rho)
    X = dec.tokens.cpu().numpy()
    rounds = int(dec.seq_rounds.cpu().numpy()[0])
    ec = O.expected_committed_iid(float(ref.alpha_mean[0]), wl.K)
    print(f"rounds {rounds} (oracle {ref.rounds[0]}), per pass {ref.rounds_per_pass[0]}, mean alpha "
          f"{ref.alpha_mean[0]:.3f}, E[C_k] {ec:.2f}, (block + n_rm) / E[C_k] = {(wl.block * 1.5) / ec:.1f}, "
          f"min margin {ref.min_margin[0]:.2e}", flush=True)
    assert int(dec.seq_pass.cpu().numpy()[0]) == 2 and np.all(X >= 0)
    if ref.min_margin[0] >= parity.TOL_CDF:
        assert np.array_equal(X[0], ref.X[0]) and rounds == ref.rounds[0]
