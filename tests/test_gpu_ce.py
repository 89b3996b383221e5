"""GPU parity of the cross-entropy use of the vocabulary head (Algorithm 1's token-level loss,
forward only, no logits written) against the oracle, through every head kernel that serves it."""
import numpy as np
import pytest
import torch

from oracle import ce_oracle as C
from paper_2605_14305_amd import binding as fb
from paper_2605_14305_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _case(R, d, V, dtype="bf16", variant=fb.FEF_GEMM_AUTO, seed=0, temperature=1.0, skip_every=0, W=None):
    W = synth.make_head(V, d, seed, dtype) if W is None else W
    sigma = 3.0 / (0.02 * np.sqrt(d))
    h = (torch.randn(R, d, generator=torch.Generator().manual_seed(seed + 1)) * sigma).to(W.dtype)
    rng = np.random.default_rng(seed)
    labels = rng.integers(0, V, size=R).astype(np.int32)
    labels[0] = 0
    labels[-1] = V - 1
    if skip_every:
        labels[::skip_every] = -1
    ce = fb.HeadCrossEntropy(R, d, V, dtype=dtype, device=DEV, gemm_variant=variant)
    ce.out_ce.fill_(-5.0)
    out, loss = ce(h.to(DEV), W.to(DEV), torch.as_tensor(labels).to(DEV), temperature=temperature)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64), float(loss.cpu()[0]), h, W, labels


def ce_tolerance(d, temperature=1.0, logit_std=3.0):
    """Bound on |CE_gpu - CE_oracle| from the arithmetic: CE = lse - L[label].
    A logit is a sum of d products that are exact in fp32 (bf16 x bf16), accumulated in fp32: d
    roundings of at most 2^-24 |partial sum| each, independent and zero-mean, partial sums below
    5 standard deviations of the scaled logit: E_L = 6 sqrt(d/3) 2^-24 (5 logit_std / tau) (six
    sigma of the accumulated rounding).  lse is 1-Lipschitz in the maximum norm, so the logit errors
    move it by at most E_L; evaluating it in fp32 (exp to 2 ulp, tree sums over V terms, log, one
    addition at |lse| < 32) and the final subtraction add less than 5e-6."""
    e_l = 6.0 * np.sqrt(d / 3.0) * 2.0 ** -24 * (5.0 * logit_std / temperature)
    return 2.0 * e_l + 5e-6


def _check(got, loss, h, W, labels, temperature=1.0, rows=None):
    rows = np.arange(len(labels)) if rows is None else rows
    want, _ = C.cross_entropy(synth.to_f64(h[rows]), synth.to_f64(W), labels[rows], temperature)
    err = np.abs(got[rows] - want)
    tol = ce_tolerance(h.shape[1], temperature)               # 4.0e-4 at d = 4096, tau = 1
    assert tol <= 5e-4 / min(1.0, temperature)
    assert np.all(err <= 2e-2 * np.abs(want) + 1e-6)          # the stated ceiling for logits and probabilities
    assert err.max() <= tol, (err.max(), tol)
    assert np.all(got[labels < 0] == 0.0)
    return want


@pytest.mark.parametrize("R,d,V,variant", [(5, 64, 1000, fb.FEF_GEMM_STREAM), (128, 256, 777, fb.FEF_GEMM_STREAM),
                                           (33, 512, 2050, fb.FEF_GEMM_AUTO), (300, 128, 999, fb.FEF_GEMM_AUTO),
                                           (129, 64, 65, fb.FEF_GEMM_TILED256), (1, 64, 1, fb.FEF_GEMM_TILED256),
                                           (700, 1024, 3001, fb.FEF_GEMM_TILED256)])
def test_cross_entropy_small_shapes(R, d, V, variant):
    got, loss, h, W, labels = _case(R, d, V, variant=variant, seed=R, skip_every=7 if R > 20 else 0)
    want = _check(got, loss, h, W, labels)
    assert abs(loss - want.sum()) <= 1e-4 * max(1.0, abs(want.sum()))
    assert abs(loss - got.sum()) <= 1e-5 * max(1.0, abs(got.sum()))   # the sum kernel adds what was written


def test_cross_entropy_f32_and_temperature():
    got, loss, h, W, labels = _case(6, 64, 32, dtype="f32", seed=3, temperature=0.7)
    _check(got, loss, h, W, labels, temperature=0.7)
    got, loss, h, W, labels = _case(40, 256, 500, seed=4, temperature=2.0)
    _check(got, loss, h, W, labels, temperature=2.0)


def test_cross_entropy_is_deterministic_and_ignores_stale_workspace():
    outs = []
    for rep in range(3):
        W = synth.make_head(3000, 512, 2)
        ce = fb.HeadCrossEntropy(200, 512, 3000, device=DEV)
        ce.workspace.fill_(rep * 91)
        h = (torch.randn(200, 512, generator=torch.Generator().manual_seed(5)) * 4).to(torch.bfloat16).to(DEV)
        lab = torch.arange(200, dtype=torch.int32, device=DEV) * 13 % 3000
        out, loss = ce(h, W.to(DEV), lab)
        torch.cuda.synchronize()
        outs.append((out.cpu().numpy().copy(), loss.cpu().numpy().copy()))
    for o in outs[1:]:
        assert np.array_equal(o[0], outs[0][0]) and np.array_equal(o[1], outs[0][1])


def test_cross_entropy_label_out_of_range_gives_nan():
    W = synth.make_head(300, 64, 1)
    ce = fb.HeadCrossEntropy(5, 64, 300, device=DEV)
    h = torch.ones(5, 64, dtype=torch.bfloat16, device=DEV)
    lab = torch.tensor([0, 299, 300, 12345, -1], dtype=torch.int32, device=DEV)
    out, loss = ce(h, W.to(DEV), lab)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert np.isfinite(o[[0, 1, 4]]).all() and o[4] == 0.0 and np.isnan(o[[2, 3]]).all()


def test_cross_entropy_llada_shape_sampled_rows():
    """LLaDA-shaped head (d=4096, V=126464), 2048 position-conditioned rows through the 256x256
    kernel and 128 through the streaming kernel; the oracle checks a seeded sample of rows."""
    wl = synth.WORKLOADS["llada_b1"]
    W = synth.make_head(wl.V, wl.d, 0, "bf16")
    for R, nsample in ((2048, 6), (128, 4)):
        got, loss, h, _, labels = _case(R, wl.d, wl.V, seed=11, W=W)
        rows = np.random.default_rng(R).choice(R, size=nsample, replace=False)
        want = _check(got, loss, h, W, labels, rows=rows)
        assert abs(loss - got.sum()) <= 1e-5 * abs(got.sum())
        print(f"R={R}: sampled CE {want.round(3).tolist()}, mean {got.mean():.3f}, log V = {np.log(wl.V):.3f}", flush=True)
