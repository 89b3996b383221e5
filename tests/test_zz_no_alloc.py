"""fef_verify_step_static (the entry point that allocates nothing and works on the library's
built-in scratch buffer) against fef_verify_step with a caller workspace: same inputs, same
kernels, so every output must be identical bit for bit.  Two calls in a row share the buffer,
the second with a smaller input, so stale contents of the first must not leak into it.  The
first call is also compared with the CPU oracle."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import fef_oracle as O
from paper_2605_14305_amd import binding as fb
from paper_2605_14305_amd import synth
import parity

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _np(t):
    return t.detach().cpu().numpy()


def _both(B, K, block, d, V, seed, step, variant=fb.FEF_GEMM_AUTO, check_oracle=False):
    """One round through both entry points; returns the static call's outputs."""
    W = synth.make_head(V, d, seed)
    hd, ht = synth.make_hidden(B, K, d, seed, 0.9, 3.0 / (0.02 * np.sqrt(d)), "bf16", 0, step)
    Wd, hdd, htd = W.to(DEV), hd.to(DEV), ht.to(DEV)
    ref_vs = fb.VerifyStep(B, K, block, d, V, device=DEV, diag=True, gemm_variant=variant)
    tok_r, acc_r, rem_r = (_np(t).copy() for t in ref_vs(hdd, htd, Wd, seed, step=step))
    diag_r = {k: _np(v).copy() for k, v in ref_vs.diag.items()}

    st_vs = fb.VerifyStep(B, K, block, d, V, device=DEV, diag=True, gemm_variant=variant)
    for t in (st_vs.out_tokens, st_vs.out_accept_len, st_vs.out_remask, *st_vs.diag.values()):
        t.fill_(-7)                       # whatever is compared below was written by the static call
    p = st_vs._params(step=step)
    assert fb.fef_workspace_bytes(p, K, block) <= fb.FEF_STATIC_SCRATCH_BYTES
    p.workspace, p.workspace_bytes = None, 0          # ignored by the static entry point
    p.stream = torch.cuda.current_stream().cuda_stream
    print(f"static call B={B} K={K} d={d} V={V} seed={seed} step={step} variant={variant}", flush=True)
    fb.fef_verify_step_static(p, hdd, htd, Wd, K, block, seed, st_vs.out_tokens, st_vs.out_accept_len,
                              st_vs.out_remask)
    torch.cuda.synchronize()
    tok, acc, rem = _np(st_vs.out_tokens), _np(st_vs.out_accept_len), _np(st_vs.out_remask)
    assert np.array_equal(tok, tok_r) and np.array_equal(acc, acc_r) and np.array_equal(rem, rem_r)
    for k, v in st_vs.diag.items():
        assert np.array_equal(_np(v).view(np.int32), diag_r[k].view(np.int32)), k
    if check_oracle:
        ref = O.verify_step(synth.to_f64(hd), synth.to_f64(ht), synth.to_f64(W), K, block, seed, step=step)
        st = parity.compare(ref, tok, acc, rem, {k: _np(v) for k, v in st_vs.diag.items()})
        assert st["near_flipped"] == 0
    return tok, acc, rem


def test_static_scratch_two_calls_second_smaller():
    # 48 rows of 20011 tokens through the streaming head kernel, then 12 rows of 5003 through the skinny one
    _both(3, 8, 32, 512, 20011, seed=5, step=0, check_oracle=True)
    _both(1, 6, 16, 512, 5003, seed=6, step=1, check_oracle=True)
    # and the first shape again: the buffer now holds the smaller call's leftovers
    _both(3, 8, 32, 512, 20011, seed=5, step=2)


def test_static_scratch_rejects_oversized_call_and_split_phases():
    B, K, block, d, V = 1, 8, 32, 512, 9000
    W = synth.make_head(V, d, 1).to(DEV)
    hd, ht = (t.to(DEV) for t in synth.make_hidden(B, K, d, 1, 0.9, 3.0 / (0.02 * np.sqrt(d)), "bf16", 0, 0))
    vs = fb.VerifyStep(B, K, block, d, V, device=DEV)
    tok_r, acc_r, rem_r = (_np(t).copy() for t in vs(hd, ht, W, 1))
    # draft call, then target call, both on the built-in buffer (the target call reads what the draft call left)
    p = vs._params()
    p.stream = torch.cuda.current_stream().cuda_stream
    p.phase = fb.FEF_PHASE_DRAFT
    drafts = torch.empty(B, K, dtype=torch.int32, device=DEV)
    fb.fef_verify_step_static(p, hd, None, W, K, block, 1, drafts, None, None)
    p.phase = fb.FEF_PHASE_TARGET
    vs.out_tokens.fill_(-7)
    fb.fef_verify_step_static(p, None, ht, W, K, block, 1, vs.out_tokens, vs.out_accept_len, vs.out_remask)
    torch.cuda.synchronize()
    assert np.array_equal(_np(vs.out_tokens), tok_r) and np.array_equal(_np(vs.out_accept_len), acc_r)
    assert np.array_equal(_np(vs.out_remask), rem_r)
    # a call that needs more than the built-in buffer is refused on the host; nothing is launched
    big = fb.make_params(64, 4096, 126464)
    assert fb.fef_workspace_bytes(big, 16, 32) > fb.FEF_STATIC_SCRATCH_BYTES
    s = fb.lib().fef_verify_step_static(ctypes.byref(big), ctypes.c_void_p(hd.data_ptr()), ctypes.c_void_p(ht.data_ptr()),
                                        ctypes.c_void_p(W.data_ptr()), 16, 32, ctypes.c_uint64(0),
                                        ctypes.c_void_p(vs.out_tokens.data_ptr()),
                                        ctypes.c_void_p(vs.out_accept_len.data_ptr()),
                                        ctypes.c_void_p(vs.out_remask.data_ptr()))
    assert s == fb.FEF_ERR_WORKSPACE and "built-in buffer" in fb.fef_last_error()
