"""GPU parity: the HIP verify step, called through the C ABI, against the CPU oracle on the
same seeded inputs (see tests/parity.py for the comparison protocol and tolerances)."""
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


def run_case(B, K, block, d, V, dtype="bf16", seed=0, rho=0.9, logit_std=3.0, variant=fb.FEF_GEMM_AUTO,
             temperature=1.0, step=0, seq_base=0, pos_base=0, n_rm=-1, final_pass=False, lowconf_scope=0,
             mask=None, pass_mask=None, conf=None, draft_tokens=None, with_logits=True, W=None,
             hidden=None, logit_atol=2e-4, recorrupt_prob=1.0, greedy=False):
    wl_sigma = logit_std / (0.02 * np.sqrt(d)) if logit_std > 0 else 1.0
    if W is None:
        W = synth.make_head(V, d, seed, dtype)
    hd, ht = hidden if hidden is not None else synth.make_hidden(B, K, d, seed, rho, wl_sigma, dtype, 0, step)
    vs = fb.VerifyStep(B, K, block, d, V, dtype=dtype, device=DEV, diag=True, diag_logits=with_logits,
                       gemm_variant=variant)
    dev = lambda a, dt: None if a is None else torch.as_tensor(np.ascontiguousarray(a), dtype=dt).to(DEV)
    g_mask, g_pm, g_cf = dev(mask, torch.uint8), dev(pass_mask, torch.uint8), dev(conf, torch.float32)
    g_dt = dev(draft_tokens, torch.int32)
    tok, acc, rem = vs(hd.to(DEV), ht.to(DEV), W.to(DEV), seed, temperature=temperature, step=step,
                       seq_base=seq_base, pos_base=pos_base, n_rm=n_rm, final_pass=final_pass,
                       lowconf_scope=lowconf_scope, mask_in=g_mask, pass_mask=g_pm, conf=g_cf,
                       draft_tokens=g_dt, recorrupt_prob=recorrupt_prob, greedy=greedy)
    torch.cuda.synchronize()
    ref = O.verify_step(synth.to_f64(hd), synth.to_f64(ht), synth.to_f64(W), K, block, seed,
                        temperature=temperature, step=step, seq_base=seq_base, pos_base=pos_base,
                        n_rm=n_rm, final_pass=final_pass, lowconf_scope=lowconf_scope, mask_in=mask,
                        pass_mask=pass_mask, conf=None if conf is None else np.asarray(conf, np.float32),
                        draft_tokens=draft_tokens, return_logits=with_logits, recorrupt_prob=recorrupt_prob,
                        greedy=greedy)
    diag = {k: _np(v) for k, v in vs.diag.items()}
    stats = parity.compare(ref, _np(tok), _np(acc), _np(rem), diag, drafts_given=draft_tokens is not None,
                           logit_atol=logit_atol)
    out = {"tokens": _np(tok), "accept_len": _np(acc), "remask": _np(rem), "diag": diag,
           "pass_mask": None if g_pm is None else _np(g_pm), "conf": None if g_cf is None else _np(g_cf)}
    return ref, out, stats


def _check_state(ref, out):
    """in/out state arrays after a compared call."""
    if out["pass_mask"] is not None:
        assert np.array_equal(out["pass_mask"], ref.pass_mask)
    if out["conf"] is not None:
        assert np.allclose(out["conf"], ref.conf, rtol=2e-4, atol=1e-12)


def test_tiny_configuration_f32_all_blocks_and_steps():
    """Tiny instance: batch 1, block 8, K=4, d=64, V=32 and V=8, fp32 head, seed 0."""
    for name in ("tiny", "tiny_v8"):
        wl = synth.WORKLOADS[name]
        W = synth.make_head(wl.V, wl.d, 0, "f32")
        total = {"near_margin": 0, "near_flipped": 0, "equal": 0}
        for blk in range(wl.gen_len // wl.block):
            for step in range(16):
                hidden = synth.make_round(wl, 0, blk, step)
                ref, out, st = run_case(wl.B, wl.K, wl.block, wl.d, wl.V, "f32", seed=0, W=W, hidden=hidden,
                                        step=step, pos_base=blk * wl.block, logit_atol=1e-5)
                for k in total:
                    total[k] += st[k]
        assert total["near_flipped"] == 0 and total["equal"] == 32


def test_tiny_scaled_logits_exercise_rejections():
    # the stated tiny scale (logit std ~0.16) almost never rejects; a wider one does
    rej = 0
    for step in range(12):
        ref, out, st = run_case(4, 4, 8, 64, 32, "f32", seed=3, rho=0.5, logit_std=2.0, step=step)
        rej += int((ref.accept_len < ref.window).sum())
        assert st["near_flipped"] == 0
    assert rej > 10


@pytest.mark.parametrize("K,V", [(8, 1000), (5, 4099), (8, 16), (3, 7)])
def test_skinny_kernel_small_shapes(K, V):
    near = 0
    for step in range(4):
        ref, out, st = run_case(1, K, 16, 512, V, seed=11, rho=0.8, step=step, variant=fb.FEF_GEMM_SKINNY)
        near += st["near_flipped"]
    assert near == 0


@pytest.mark.parametrize("B,K,V", [(1, 16, 1000), (2, 8, 4099), (3, 5, 16), (1, 9, 7), (2, 7, 10300)])
def test_skinny_kernel_two_row_groups(B, K, V):
    """17..32 rows through the head: the streaming kernel with two resident 16-row groups."""
    near = 0
    for step in range(3):
        ref, out, st = run_case(B, K, 16, 512, V, seed=15, rho=0.8, step=step, variant=fb.FEF_GEMM_SKINNY)
        near += st["near_flipped"]
    assert near == 0


@pytest.mark.parametrize("B,K,d,V", [(1, 8, 1024, 3000), (2, 8, 2048, 1500), (1, 16, 2560, 2000), (1, 5, 3072, 1001),
                                     (2, 4, 3584, 777)])
def test_skinny_kernel_other_hidden_sizes(B, K, d, V):
    """Every hidden size the streaming kernels for at most 32 rows are instantiated for (d = 256 KS),
    with 16 rows or fewer and with 17 to 32; AUTO must pick them."""
    p = fb.make_params(B, d, V)
    assert fb.fef_select_gemm(p, K) == fb.FEF_GEMM_SKINNY
    near = 0
    for step in range(2):
        ref, out, st = run_case(B, K, 16, d, V, seed=19, rho=0.8, step=step)
        near += st["near_flipped"]
    assert near == 0
    assert fb.fef_select_gemm(fb.make_params(B, d + 64, V), K) == fb.FEF_GEMM_STREAM     # no instantiation: streaming kernel


def test_window_16_batch1_full_size(llada_head):
    """LLaDA-shaped head with a 16-token window at batch 1 (32 rows through the head), every
    output element against the oracle."""
    wl, W, Wd, W64 = llada_head
    K, block = 16, 32
    vs = fb.VerifyStep(1, K, block, wl.d, wl.V, device=DEV, diag=True, diag_logits=True)
    assert fb.fef_select_gemm(vs._params(), K) == fb.FEF_GEMM_SKINNY
    near = compared = 0
    for step in range(2):
        hd, ht = synth.make_hidden(1, K, wl.d, 4, wl.rho, wl.sigma_h, "bf16", 0, step)
        tok, acc, rem = vs(hd.to(DEV), ht.to(DEV), Wd, 4, step=step)
        torch.cuda.synchronize()
        ref = O.verify_step(synth.to_f64(hd), synth.to_f64(ht), W64, K, block, 4, step=step, return_logits=True)
        st = parity.compare(ref, _np(tok), _np(acc), _np(rem), {k: _np(v) for k, v in vs.diag.items()})
        near += st["near_flipped"]; compared += st["equal"]
        print(f"step {step}: accept_len {ref.accept_len[0]} {st}", flush=True)
    assert compared >= 1 and near <= 1


@pytest.mark.parametrize("B,K,d,V", [(5, 8, 64, 1000), (20, 8, 512, 777), (3, 16, 3584, 2050),
                                     (70, 2, 128, 300), (1, 1, 64, 1)])
def test_tiled_kernel_small_shapes(B, K, d, V):
    ref, out, st = run_case(B, K, max(K, 16), d, V, seed=12, rho=0.8, variant=fb.FEF_GEMM_TILED)
    assert st["near_flipped"] <= B // 20


@pytest.mark.parametrize("B,K,d,V", [(5, 8, 64, 1000), (20, 8, 512, 777), (40, 4, 128, 2050), (1, 1, 64, 1),
                                     (17, 16, 256, 300), (32, 8, 192, 515), (70, 8, 128, 520)])
def test_tiled256_kernel_small_shapes(B, K, d, V):
    """Up to 256 rows: eight wavefronts of 128 x 64; above: four of 128 x 128 (320 and 544 rows: a last
    row tile with wavefronts that have no rows; 512: two full row tiles; 1120: five)."""
    ref, out, st = run_case(B, K, max(K, 16), d, V, seed=13, rho=0.8, variant=fb.FEF_GEMM_TILED256)
    assert st["near_flipped"] <= B // 20


@pytest.mark.parametrize("B,K,d,V", [(5, 8, 64, 1000), (3, 5, 128, 777), (8, 8, 512, 2050), (1, 1, 64, 1),
                                     (4, 16, 256, 300), (2, 9, 3584, 1500), (6, 8, 1024, 513), (7, 8, 512, 2049),
                                     (4, 8, 256, 600), (3, 11, 128, 520)])
def test_stream_kernel_small_shapes(B, K, d, V):
    """Persistent workgroups of 64 rows (M <= 64) or 128 rows x 256 tokens: 2 to 128 rows through the
    head including M = 64 and 66 on either side of the switch, k loops of 2 to 112 steps (prologue only,
    tail only, steady steps plus tail) each started at another k-step and wrapped, ragged V."""
    ref, out, st = run_case(B, K, max(K, 16), d, V, seed=16, rho=0.8, variant=fb.FEF_GEMM_STREAM)
    assert st["near_flipped"] <= B // 20


@pytest.mark.parametrize("B,K,d,V", [(5, 8, 512, 1000), (4, 5, 512, 777), (8, 8, 512, 2050), (17, 1, 512, 1),
                                     (4, 16, 1024, 300), (2, 9, 3584, 1500), (6, 8, 1024, 513), (7, 8, 512, 2049),
                                     (3, 16, 512, 40000), (5, 8, 1536, 33000), (2, 16, 512, 16 * 2048 + 5)])
def test_rowstream_kernel_small_shapes(B, K, d, V):
    """The kernel that streams W into registers (33 to 128 rows, d a multiple of 512): the three
    stage heights (64, 96, 128 rows), one to seven macro-steps rounds per tile, fewer tiles than
    wavefronts (empty runs), runs of unequal length inside a workgroup, ragged last tile."""
    M = 2 * B * K   # AUTO: where this kernel needs fewer rows (64 / 96 / 128) than the LDS-streaming one (64 / 128)
    want = fb.FEF_GEMM_ROWSTREAM if M <= 48 or 64 < M <= 96 else fb.FEF_GEMM_STREAM
    assert fb.fef_select_gemm(fb.make_params(B, d, V), K) == want
    flipped = 0
    for step in range(2):
        ref, out, st = run_case(B, K, max(K, 16), d, V, seed=23, rho=0.8, step=step, variant=fb.FEF_GEMM_ROWSTREAM)
        flipped += st["near_flipped"]
    assert flipped <= max(1, B // 10)
    ref, out, st = run_case(B, K, max(K, 16), d, V, seed=23, rho=0.9, step=4, variant=fb.FEF_GEMM_ROWSTREAM, greedy=True,
                            temperature=0.7)
    assert st["near_flipped"] <= max(1, B // 10)


@pytest.mark.parametrize("B,variant", [(3, fb.FEF_GEMM_AUTO), (4, fb.FEF_GEMM_AUTO), (6, fb.FEF_GEMM_AUTO),
                                       (8, fb.FEF_GEMM_AUTO), (8, fb.FEF_GEMM_ROWSTREAM), (4, fb.FEF_GEMM_ROWSTREAM)])
def test_llada_shape_through_the_streaming_kernels(llada_head, B, variant):
    """B = 3, 4, 6, 8 at full d and V (48, 64, 96, 128 rows through the head): AUTO gives 48 and 96 to the
    row-streaming kernel and 64 and 128 to the LDS-streaming one; the row-streaming kernel also on the sizes
    AUTO gives the other.  The oracle checks a seeded subset of sequences."""
    wl, W, Wd, W64 = llada_head
    K, block = 8, 32
    vs = fb.VerifyStep(B, K, block, wl.d, wl.V, device=DEV, diag=True, gemm_variant=variant)
    want = {fb.FEF_GEMM_AUTO: fb.FEF_GEMM_ROWSTREAM if B in (3, 6) else fb.FEF_GEMM_STREAM}.get(variant, variant)
    assert fb.fef_select_gemm(vs._params(), K) == want
    hd, ht = synth.make_hidden(B, K, wl.d, 9, wl.rho, wl.sigma_h, "bf16", 0, 2)
    tok, acc, rem = vs(hd.to(DEV), ht.to(DEV), Wd, 9, step=2)
    torch.cuda.synchronize()
    equal = near = 0
    for b in [0, B // 2, B - 1]:
        r = O.verify_step(synth.to_f64(hd[b:b + 1]), synth.to_f64(ht[b:b + 1]), W64, K, block, 9, step=2,
                          seq_base=b)
        diag = {k: _np(v)[b:b + 1] if k != "lse" else _np(v)[:, b:b + 1] for k, v in vs.diag.items()}
        st = parity.compare(r, _np(tok)[b:b + 1], _np(acc)[b:b + 1], _np(rem)[b:b + 1], diag)
        equal += st["equal"]; near += st["near_margin"]
        print(f"seq {b}: {st}", flush=True)
    print(f"B={B}: {equal} of 3 sampled sequences identical, {near} near-margin", flush=True)
    assert equal >= 2


def test_maximum_window_and_block():
    """K = 64 (the largest window) in a block of 4096 positions (the largest block): window slots by
    rank over a long mask, LowConf ranking over 4096 candidates, both scopes."""
    B, K, block, d, V = 3, 64, 4096, 64, 300
    rng = np.random.default_rng(2)
    mask = np.zeros((B, block), np.uint8)
    mask[0, rng.choice(block, size=40, replace=False)] = 1          # fewer than K unresolved: resolves now
    mask[1, rng.choice(block, size=500, replace=False)] = 1
    mask[2, :] = 1
    pm = ((1 - mask) * (rng.random((B, block)) < 0.5)).astype(np.uint8)
    conf = rng.random((B, block)).astype(np.float32)
    for scope, n_rm in ((0, 1000), (1, -1)):
        ref, out, st = run_case(B, K, block, d, V, seed=60 + scope, rho=0.999, logit_std=1.0, mask=mask, pass_mask=pm,
                                conf=conf, n_rm=n_rm, lowconf_scope=scope, with_logits=False)
        assert st["near_flipped"] == 0
        if st["remask_skipped"] == 0:
            _check_state(ref, out)
        assert ref.window.tolist() == [40, 64, 64]


def test_empty_windows_and_many_sequences():
    """300 one-token windows, a third of them with nothing left to resolve (empty window: outputs -1,
    accepted length 0, mask unchanged; with state given, LowConf still fires on a resolved block)."""
    B, K, block, d, V = 300, 1, 4, 64, 50
    rng = np.random.default_rng(3)
    mask = (rng.random((B, block)) < 0.4).astype(np.uint8)
    mask[::3] = 0
    ref, out, st = run_case(B, K, block, d, V, seed=70, rho=0.7, mask=mask, final_pass=True, with_logits=False,
                            variant=fb.FEF_GEMM_TILED256)
    assert st["near_flipped"] <= 3
    empty = mask.sum(1) == 0
    assert empty.sum() >= 100 and np.all(out["tokens"][empty] == -1) and np.all(out["accept_len"][empty] == 0)
    assert np.all(out["remask"][empty] == 0)


def test_very_large_vocabulary_generic_partial_merge():
    # more than 2560 partial tiles and 1024 residual chunks per row: the memory-resident code paths
    ref, out, st = run_case(2, 2, 16, 64, 270001, seed=14, rho=0.8, variant=fb.FEF_GEMM_TILED, with_logits=False)
    assert st["near_flipped"] == 0 and st["equal"] == 2


@pytest.mark.parametrize("B,K,d,variant", [(1, 8, 512, fb.FEF_GEMM_SKINNY), (5, 8, 64, fb.FEF_GEMM_STREAM)])
def test_workgroup_shares_of_more_than_640_tokens(B, K, d, variant):
    """One partial per row and workgroup over its contiguous share of the vocabulary (the kernels up to 32 rows, the
    LDS-streaming kernel): with 170003 tokens over 256 workgroups a share has 656 to 672 tokens, more than the
    draft sampler keeps in registers, so the selected share is re-read from the logits."""
    ref, out, st = run_case(B, K, 16, d, 170003, seed=15, rho=0.8, variant=variant, with_logits=False)
    assert st["near_flipped"] <= B // 20 and st["equal"] + st["near_margin"] >= B


def test_skinny_and_tiled_agree():
    W = synth.make_head(3000, 512, 5)
    hidden = synth.make_hidden(1, 8, 512, 5, 0.7, 3.0 / (0.02 * np.sqrt(512)))
    a = run_case(1, 8, 32, 512, 3000, seed=5, W=W, hidden=hidden, variant=fb.FEF_GEMM_SKINNY)
    b = run_case(1, 8, 32, 512, 3000, seed=5, W=W, hidden=hidden, variant=fb.FEF_GEMM_TILED)
    assert np.abs(a[1]["diag"]["logits"] - b[1]["diag"]["logits"]).max() < 1e-4
    if a[2]["near_flipped"] == 0 and b[2]["near_flipped"] == 0:
        assert np.array_equal(a[1]["tokens"], b[1]["tokens"])


def test_deterministic_bits():
    W = synth.make_head(5000, 512, 1).to(DEV)
    hd, ht = (t.to(DEV) for t in synth.make_hidden(2, 4, 512, 1, 0.8, 3.0 / (0.02 * np.sqrt(512))))
    for variant in (fb.FEF_GEMM_SKINNY, fb.FEF_GEMM_TILED, fb.FEF_GEMM_TILED256, fb.FEF_GEMM_STREAM, fb.FEF_GEMM_ROWSTREAM):
        outs = []
        for rep in range(3):
            vs = fb.VerifyStep(2, 4, 8, 512, 5000, diag=True, diag_logits=True, gemm_variant=variant)
            vs.workspace.fill_(rep * 37)        # stale workspace contents must not matter
            tok, acc, rem = vs(hd, ht, W, 42, step=9)
            torch.cuda.synchronize()
            outs.append((_np(tok).copy(), _np(acc).copy(), _np(rem).copy(), _np(vs.diag["logits"]).copy(),
                         _np(vs.diag["alpha"]).copy()))
        for o in outs[1:]:
            for x, y in zip(o, outs[0]):
                assert np.array_equal(x, y)


def test_temperature_step_and_bases():
    ref, out, st = run_case(3, 4, 16, 512, 2000, seed=21, temperature=0.5, step=77, seq_base=1000,
                            pos_base=4096, rho=0.95, variant=fb.FEF_GEMM_TILED)
    assert st["near_flipped"] == 0
    # batch invariance on the device: sequence 2 alone, addressed by seq_base, gives the same row
    W = synth.make_head(2000, 512, 21)
    hd, ht = synth.make_hidden(3, 4, 512, 21, 0.95, 3.0 / (0.02 * np.sqrt(512)), "bf16", 0, 77)
    ref1, out1, st1 = run_case(1, 4, 16, 512, 2000, seed=21, temperature=0.5, step=77, seq_base=1002,
                               pos_base=4096, W=W, hidden=(hd[2:3].contiguous(), ht[2:3].contiguous()),
                               variant=fb.FEF_GEMM_TILED)
    assert np.array_equal(out1["tokens"][0], out["tokens"][2])
    assert out1["accept_len"][0] == out["accept_len"][2]


def test_masks_window_boundary_and_supplied_drafts():
    B, K, block, d, V = 6, 4, 8, 512, 600
    mask = np.array([[1, 1, 1, 1, 1, 1, 1, 1],
                     [0, 0, 1, 0, 1, 0, 0, 1],
                     [0, 0, 0, 0, 0, 0, 1, 0],
                     [0, 0, 0, 0, 0, 0, 0, 0],
                     [1, 0, 1, 0, 1, 0, 1, 0],
                     [0, 1, 1, 1, 1, 1, 1, 1]], np.uint8)
    ref, out, st = run_case(B, K, block, d, V, seed=31, rho=0.6, mask=mask, final_pass=True,
                            pass_mask=np.zeros((B, block), np.uint8), conf=np.zeros((B, block), np.float32))
    assert ref.window.tolist() == [4, 3, 1, 0, 4, 4]
    assert st["near_flipped"] == 0
    _check_state(ref, out)
    drafts = np.random.default_rng(0).integers(0, V, size=(B, K)).astype(np.int32)
    ref, out, st = run_case(B, K, block, d, V, seed=31, rho=0.6, mask=mask, draft_tokens=drafts)
    assert np.array_equal(out["diag"]["draft_tokens"][ref.slot_pos >= 0], drafts[ref.slot_pos >= 0])
    assert st["near_flipped"] == 0


@pytest.mark.parametrize("scope", [0, 1])
def test_low_confidence_remask_fires_when_block_resolves(scope):
    B, K, block, d, V = 8, 4, 8, 512, 500
    rng = np.random.default_rng(5)
    mask = np.zeros((B, block), np.uint8)
    pm = np.zeros((B, block), np.uint8)
    for b in range(B):
        unresolved = rng.choice(block, size=1 + b % 3, replace=False)   # 1..3 left: may resolve now
        mask[b, unresolved] = 1
        pm[b, rng.choice(np.setdiff1d(np.arange(block), unresolved), size=3, replace=False)] = 1
    conf = rng.random((B, block)).astype(np.float32)
    fired = 0
    for n_rm in (-1, 2, 0, 100):
        ref, out, st = run_case(B, K, block, d, V, seed=41, rho=0.9, mask=mask, pass_mask=pm, conf=conf,
                                n_rm=n_rm, lowconf_scope=scope)
        resolved = (ref.remask.sum(1) > 0) & ((mask.sum(1) - ref.committed) == 0)
        fired += int(resolved.sum())
        if st["near_flipped"] == 0 and st["remask_skipped"] == 0:
            _check_state(ref, out)
    assert fired > 0
    ref, out, st = run_case(B, K, block, d, V, seed=41, rho=0.9, mask=mask, pass_mask=pm, conf=conf,
                            n_rm=3, lowconf_scope=scope, final_pass=True)
    assert np.all(out["remask"] <= mask)


def test_stochastic_recorruption_of_the_low_confidence_selection():
    """Re-corruption through the absorbing kernel with probability < 1: the re-masked set is the
    oracle's (a subset of LowConf's selection chosen by Philox stream 3), everything else as before."""
    B, K, block, d, V = 16, 4, 8, 512, 500
    rng = np.random.default_rng(6)
    mask = np.zeros((B, block), np.uint8)
    mask[:, 5] = 1                                       # one position left: this round resolves the block
    pm = np.ones((B, block), np.uint8) - mask
    conf = rng.random((B, block)).astype(np.float32)
    counts = {}
    for prob in (1.0, 0.7, 0.3, 5e-8):
        ref, out, st = run_case(B, K, block, d, V, seed=43, rho=0.9, mask=mask, pass_mask=pm, conf=conf,
                                n_rm=6, recorrupt_prob=prob, step=3, pos_base=64, seq_base=5)
        assert st["near_flipped"] == 0 and st["remask_skipped"] == 0
        _check_state(ref, out)
        assert np.array_equal(out["remask"], ref.remask)
        counts[prob] = int(out["remask"].sum())
    assert counts[1.0] == 6 * B and counts[5e-8] == 0
    assert counts[1.0] > counts[0.7] > counts[0.3] > 0


@pytest.mark.parametrize("B,K,d,V,variant", [(1, 8, 512, 3000, fb.FEF_GEMM_SKINNY), (2, 8, 512, 5003, fb.FEF_GEMM_SKINNY),
                                             (6, 8, 256, 1500, fb.FEF_GEMM_STREAM), (24, 4, 128, 999, fb.FEF_GEMM_TILED256),
                                             (5, 4, 64, 700, fb.FEF_GEMM_TILED), (3, 4, 64, 40, fb.FEF_GEMM_F32)])
def test_greedy_variant(B, K, d, V, variant):
    """Zero-temperature variant: arg max drafts, accept on equal arg maxes, corrected token =
    target arg max, confidences from the finite-temperature softmax; every head kernel's partials."""
    dtype = "f32" if variant == fb.FEF_GEMM_F32 else "bf16"
    acc_lens, flipped = [], 0
    for step, rho in enumerate((0.99, 0.9, 0.6)):
        ref, out, st = run_case(B, K, 16, d, V, dtype, seed=51, rho=rho, step=step, variant=variant, greedy=True,
                                temperature=0.8, logit_atol=2e-4 if dtype == "bf16" else 1e-5)
        flipped += st["near_flipped"]
        acc_lens += ref.accept_len.tolist()
    assert flipped <= 1
    assert min(acc_lens) < K and max(acc_lens) > 0          # both rejections and acceptances occurred


def test_greedy_variant_with_supplied_drafts_and_no_uniforms():
    B, K, d, V = 4, 4, 512, 2000
    W = synth.make_head(V, d, 3)
    hidden = synth.make_hidden(B, K, d, 3, 0.9, 3.0 / (0.02 * np.sqrt(d)))
    a = run_case(B, K, 8, d, V, seed=1, W=W, hidden=hidden, greedy=True, step=0)
    b = run_case(B, K, 8, d, V, seed=99, W=W, hidden=hidden, greedy=True, step=7, pos_base=64)
    assert np.array_equal(a[1]["tokens"], b[1]["tokens"]) and np.array_equal(a[1]["accept_len"], b[1]["accept_len"])
    drafts = a[0].draft_tokens.copy()
    drafts[:, 1] = (drafts[:, 1] + 1) % V                       # wrong at slot 1 unless it happens to be the target's
    ref, out, st = run_case(B, K, 8, d, V, seed=1, W=W, hidden=hidden, greedy=True, draft_tokens=drafts.astype(np.int32))
    assert st["near_flipped"] == 0 and np.all(out["accept_len"] <= 1)


def test_greedy_variant_in_split_call_order():
    """DRAFT call returns the arg max drafts, TARGET call verifies them against the target arg maxes."""
    B, K, d, V, block = 5, 4, 256, 1200, 8
    W = synth.make_head(V, d, 4)
    hd, ht = synth.make_hidden(B, K, d, 4, 0.9, 3.0 / (0.02 * np.sqrt(d)))
    Wd, hdd, htd = W.to(DEV), hd.to(DEV), ht.to(DEV)
    vs = fb.VerifyStep(B, K, block, d, V, device=DEV, diag=True, diag_logits=True)
    tok, _, _ = vs(hdd, None, Wd, 2, step=1, phase=fb.FEF_PHASE_DRAFT, greedy=True)
    torch.cuda.synchronize()
    drafts = _np(tok).copy()
    tok, acc, rem = vs(None, htd, Wd, 2, step=1, phase=fb.FEF_PHASE_TARGET, greedy=True)
    torch.cuda.synchronize()
    ref = O.verify_step(synth.to_f64(hd), synth.to_f64(ht), synth.to_f64(W), K, block, 2, step=1, greedy=True,
                        return_logits=True)
    st = parity.compare(ref, _np(tok), _np(acc), _np(rem), {k: _np(v) for k, v in vs.diag.items()})
    clear = ref.argmax_gap[0] >= parity.TOL_ARGMAX
    assert np.array_equal(drafts[clear], ref.draft_tokens[clear]) and st["near_flipped"] == 0


def test_stateful_pass_over_a_block_matches_oracle():
    """Rounds chained through mask / pass_mask / conf on each side separately until the block
    resolves and LowConf fires; then a second pass over the re-masked positions."""
    B, K, block, d, V = 4, 4, 16, 512, 800
    W = synth.make_head(V, d, 7)
    Wd, W64 = W.to(DEV), synth.to_f64(W)
    vs = fb.VerifyStep(B, K, block, d, V, device=DEV, diag=True)
    g_mask = torch.ones(B, block, dtype=torch.uint8, device=DEV)
    g_pm = torch.zeros(B, block, dtype=torch.uint8, device=DEV)
    g_cf = torch.zeros(B, block, dtype=torch.float32, device=DEV)
    o_mask, o_pm, o_cf = np.ones((B, block), np.uint8), np.zeros((B, block), np.uint8), np.zeros((B, block))
    alive = np.ones(B, bool)          # sequences still in lock-step with the oracle
    sigma = 3.0 / (0.02 * np.sqrt(d))
    refired = 0
    for step in range(24):
        hd, ht = synth.make_hidden(B, K, d, 7, 0.85, sigma, "bf16", 0, step)
        tok, acc, rem = vs(hd.to(DEV), ht.to(DEV), Wd, 7, step=step, mask_in=g_mask, pass_mask=g_pm,
                           conf=g_cf, n_rm=5)
        torch.cuda.synchronize()
        ref = O.verify_step(synth.to_f64(hd), synth.to_f64(ht), W64, K, block, 7, step=step, mask_in=o_mask,
                            pass_mask=o_pm, conf=o_cf, n_rm=5)
        st = parity.compare(ref, _np(tok), _np(acc), _np(rem))
        for b in range(B):
            near = (ref.draft_gap[b] < parity.TOL_CDF).any() or (ref.accept_margin[b] < parity.TOL_ACCEPT).any() \
                or ref.resid_gap[b] < parity.TOL_CDF or ref.lowconf_gap[b] < parity.TOL_CONF
            if near:
                alive[b] = False
            if alive[b]:
                assert np.array_equal(_np(rem)[b], ref.remask[b])
                assert np.array_equal(_np(g_pm)[b], ref.pass_mask[b])
                assert np.allclose(_np(g_cf)[b], ref.conf[b], rtol=2e-4, atol=1e-12)
                refired += int(o_mask[b].sum() - ref.committed[b] == 0)
        g_mask = rem.clone()
        o_mask, o_pm, o_cf = ref.remask, ref.pass_mask, ref.conf
        # keep dropped sequences from drifting: re-seed their device state from the oracle's
        for b in np.flatnonzero(~alive):
            g_mask[b] = torch.as_tensor(o_mask[b]).to(DEV)
            g_pm[b] = torch.as_tensor(o_pm[b]).to(DEV)
            g_cf[b] = torch.as_tensor(o_cf[b].astype(np.float32)).to(DEV)
            alive[b] = True
    assert refired >= B          # every sequence resolved its block at least once


@pytest.fixture(scope="module")
def llada_head():
    wl = synth.WORKLOADS["llada_b1"]
    W = synth.make_head(wl.V, wl.d, 0, "bf16")
    return wl, W, W.to(DEV), synth.to_f64(W)


def test_llada_shape_batch1_full_size(llada_head):
    """LLaDA-8B-shaped single sequence (d=4096, V=126464, K=8, block 32) in the configuration
    the benchmark times, every element of the outputs against the oracle."""
    wl, W, Wd, W64 = llada_head
    vs = fb.VerifyStep(wl.B, wl.K, wl.block, wl.d, wl.V, device=DEV, diag=True, diag_logits=True)
    assert fb.fef_select_gemm(vs._params(), wl.K) == fb.FEF_GEMM_SKINNY
    near = compared = 0
    acc_lens = []
    for step in range(6):
        hd, ht = synth.make_round(wl, 0, block_index=step % 2, step=step)
        tok, acc, rem = vs(hd.to(DEV), ht.to(DEV), Wd, 0, step=step, pos_base=32 * (step % 2))
        torch.cuda.synchronize()
        ref = O.verify_step(synth.to_f64(hd), synth.to_f64(ht), W64, wl.K, wl.block, 0, step=step,
                            pos_base=32 * (step % 2), return_logits=True)
        st = parity.compare(ref, _np(tok), _np(acc), _np(rem), {k: _np(v) for k, v in vs.diag.items()})
        near += st["near_flipped"]; compared += st["equal"]
        acc_lens.append(int(ref.accept_len[0]))
        print(f"step {step}: accept_len {ref.accept_len[0]} alpha {ref.alpha[0].round(3)} {st}", flush=True)
    assert compared >= 5 and near <= 1
    assert 0 < np.mean(acc_lens) < wl.K       # the recipe gives a mix of acceptances and rejections


def test_llada_shape_batched_subset(llada_head):
    """B=16 at full d and V through the tiled kernel; the oracle checks a seeded subset of
    sequences, which is valid because a sequence's outcome depends only on its own rows and
    (seed, sequence id, step, position)."""
    wl, W, Wd, W64 = llada_head
    B, K, block = 16, 8, 32
    vs = fb.VerifyStep(B, K, block, wl.d, wl.V, device=DEV, diag=True)
    hd, ht = synth.make_hidden(B, K, wl.d, 3, wl.rho, wl.sigma_h, "bf16", 0, 5)
    tok, acc, rem = vs(hd.to(DEV), ht.to(DEV), Wd, 3, step=5)
    torch.cuda.synchronize()
    # sequence ids differ per picked row, so the oracle runs them one at a time with seq_base
    equal = near = 0
    for b in [0, 7, 15]:
        r = O.verify_step(synth.to_f64(hd[b:b + 1]), synth.to_f64(ht[b:b + 1]), W64, K, block, 3, step=5,
                          seq_base=b)
        diag = {k: _np(v)[b:b + 1] if k != "lse" else _np(v)[:, b:b + 1] for k, v in vs.diag.items()}
        st = parity.compare(r, _np(tok)[b:b + 1], _np(acc)[b:b + 1], _np(rem)[b:b + 1], diag)
        equal += st["equal"]; near += st["near_margin"]
        print(f"seq {b}: {st}", flush=True)
    print(f"{equal} of 3 sampled sequences identical, {near} near-margin", flush=True)
    assert equal >= 2


def test_dream_shape_subset():
    """Dream-7B-shaped rows (d=3584, V=151936, K=16) through both bf16 kernels."""
    wl = synth.WORKLOADS["dream_b32"]
    W = synth.make_head(wl.V, wl.d, 1, "bf16")
    Wd, W64 = W.to(DEV), synth.to_f64(W)
    B = 4
    vs = fb.VerifyStep(B, wl.K, wl.block, wl.d, wl.V, device=DEV, diag=True)
    hd, ht = synth.make_round(wl, 1, 0, 2, B=B)
    tok, acc, rem = vs(hd.to(DEV), ht.to(DEV), Wd, 1, step=2)
    torch.cuda.synchronize()
    ref = O.verify_step(synth.to_f64(hd), synth.to_f64(ht), W64, wl.K, wl.block, 1, step=2)
    st = parity.compare(ref, _np(tok), _np(acc), _np(rem), {k: _np(v) for k, v in vs.diag.items()})
    print(st, flush=True)
    assert st["equal"] >= 3
    # skinny kernel at d=3584: one sequence, K=8
    vs1 = fb.VerifyStep(1, 8, wl.block, wl.d, wl.V, device=DEV, diag=True, gemm_variant=fb.FEF_GEMM_SKINNY)
    hd1, ht1 = hd[:1, :8].contiguous(), ht[:1, :8].contiguous()
    tok, acc, rem = vs1(hd1.to(DEV), ht1.to(DEV), Wd, 1, step=2)
    torch.cuda.synchronize()
    ref1 = O.verify_step(synth.to_f64(hd1), synth.to_f64(ht1), W64, 8, wl.block, 1, step=2)
    parity.compare(ref1, _np(tok), _np(acc), _np(rem), {k: _np(v) for k, v in vs1.diag.items()})


def test_dream_shape_window_16_batch1_full_size():
    """Dream-7B-shaped single sequence with the paper's largest window (B=1, K=16, d=3584,
    V=151936: 32 rows through the head).  AUTO gives it the 32-row streaming kernel at d=3584,
    whose per-workgroup token runs exceed 512 tokens at this V, so the draft draw inside a tile
    takes the memory-resident path.  Every output element against the oracle."""
    wl = synth.WORKLOADS["dream_b32"]
    W = synth.make_head(wl.V, wl.d, 3, "bf16")
    Wd, W64 = W.to(DEV), synth.to_f64(W)
    vs = fb.VerifyStep(1, wl.K, wl.block, wl.d, wl.V, device=DEV, diag=True, diag_logits=True)
    assert fb.fef_select_gemm(vs._params(), wl.K) == fb.FEF_GEMM_SKINNY
    equal = flipped = 0
    acc_lens = []
    for step in range(3):
        hd, ht = synth.make_round(wl, 3, block_index=step % 2, step=step, B=1)
        tok, acc, rem = vs(hd.to(DEV), ht.to(DEV), Wd, 3, step=step, pos_base=64 * (step % 2))
        torch.cuda.synchronize()
        ref = O.verify_step(synth.to_f64(hd), synth.to_f64(ht), W64, wl.K, wl.block, 3, step=step,
                            pos_base=64 * (step % 2), return_logits=True)
        st = parity.compare(ref, _np(tok), _np(acc), _np(rem), {k: _np(v) for k, v in vs.diag.items()})
        equal += st["equal"]; flipped += st["near_flipped"]
        acc_lens.append(int(ref.accept_len[0]))
        print(f"step {step}: accept_len {ref.accept_len[0]} alpha {ref.alpha[0].round(3)} {st}", flush=True)
    assert equal >= 2 and flipped <= 1
    assert st["draft_slots"] == wl.K and st["draft_near"] <= 2      # the draft draws were compared slot by slot


def test_dream_shape_full_batch_sampled():
    """Dream-7B-shaped batch at full size (B=32, K=16, d=3584, V=151936: 1024 rows through the
    256x256 MFMA kernel), launched as the benchmark launches it (no diagnostics); the oracle
    checks sampled sequences one by one."""
    wl = synth.WORKLOADS["dream_b32"]
    W = synth.make_head(wl.V, wl.d, 2, "bf16")
    Wd, W64 = W.to(DEV), synth.to_f64(W)
    vs = fb.VerifyStep(wl.B, wl.K, wl.block, wl.d, wl.V, device=DEV)
    assert fb.fef_select_gemm(vs._params(), wl.K) == fb.FEF_GEMM_TILED256
    hd, ht = synth.make_round(wl, 2, 1, 7)
    tok, acc, rem = vs(hd.to(DEV), ht.to(DEV), Wd, 2, step=7, pos_base=64)
    torch.cuda.synchronize()
    equal = 0
    for b in (0, 13, 31):
        r = O.verify_step(synth.to_f64(hd[b:b + 1]), synth.to_f64(ht[b:b + 1]), W64, wl.K, wl.block, 2, step=7,
                          seq_base=b, pos_base=64)
        st = parity.compare(r, _np(tok)[b:b + 1], _np(acc)[b:b + 1], _np(rem)[b:b + 1])
        equal += st["equal"]
        print(f"seq {b}: accept_len {r.accept_len[0]} {st}", flush=True)
    assert equal >= 2
    # whole-batch properties that hold at any size
    t, a_ = _np(tok), _np(acc)
    assert np.all((a_ >= 0) & (a_ <= wl.K))
    for b in range(wl.B):
        c = min(a_[b] + 1, wl.K)
        assert np.all((t[b, :c] >= 0) & (t[b, :c] < wl.V)) and np.all(t[b, c:] == -1)
        assert _np(rem)[b].sum() == wl.block - c


def test_acceptance_sweep_matches_theorem_2(llada_head):
    """Acceptance-rate sweep at scale (B=64, K=16, d=4096, V=126464; rho = 0.999 added to the stated
    three so that the mean overlap reaches ~0.95, where Theorem 2's E[C_16] ~ 11): for each (rho, tau) the mean
    committed length of the HIP path matches Theorem 2 evaluated on the per-slot acceptance
    probabilities alpha = sum min(p, q) that the same call reports, and sampled sequences match the
    oracle.  Prints mean alpha, mean C, E[C_k] and the idealised acceleration E[C_k]/2."""
    wl, W, Wd, W64 = llada_head
    B, K, block = 64, 16, 32
    vs = fb.VerifyStep(B, K, block, wl.d, wl.V, device=DEV, diag=True)
    alphas_seen = []
    for rho in (0.5, 0.9, 0.99, 0.999):
        for tau in (0.5, 1.0):
            C, EC, al = [], [], []
            for step in range(3):
                hd, ht = synth.make_hidden(B, K, wl.d, 5, rho, wl.sigma_h, "bf16", 0, step)
                tok, acc, rem = vs(hd.to(DEV), ht.to(DEV), Wd, 5, step=step, temperature=tau)
                torch.cuda.synchronize()
                a_, alpha = _np(acc), _np(vs.diag["alpha"]).astype(np.float64)
                C.append(np.minimum(a_ + 1, K))
                EC.append([O.expected_committed(alpha[b]) for b in range(B)])
                al.append(alpha.mean())
                if step == 0:
                    for b in (3, 60):
                        r = O.verify_step(synth.to_f64(hd[b:b + 1]), synth.to_f64(ht[b:b + 1]), W64, K, block, 5,
                                          step=step, seq_base=b, temperature=tau)
                        diag = {"alpha": alpha[b:b + 1], "resid_mass": _np(vs.diag["resid_mass"])[b:b + 1]}
                        parity.compare(r, _np(tok)[b:b + 1], a_[b:b + 1], _np(rem)[b:b + 1], diag)
            C, EC = np.concatenate(C).astype(np.float64), np.concatenate(EC)
            se = C.std() / np.sqrt(C.size) + 1e-9
            print(f"rho={rho} tau={tau}: mean alpha {np.mean(al):.3f}  mean C {C.mean():.3f}  "
                  f"Theorem-2 E[C] {EC.mean():.3f}  S=E[C]/2 {EC.mean() / 2:.3f}  (n={C.size})", flush=True)
            assert abs(C.mean() - EC.mean()) < 4 * se + 0.02
            alphas_seen.append(np.mean(al))
    assert min(alphas_seen) < 0.2 and max(alphas_seen) > 0.93     # the sweep spans the stated range of overlaps, ~0.2 to ~0.95


@pytest.mark.parametrize("B,K,d,V", [(1, 8, 512, 3000), (6, 8, 256, 2050), (40, 4, 128, 700)])
def test_separate_draft_model_head(B, K, d, V):
    """Ablation 3's "A / B" setting: the DRAFT call projects with the draft model's own output
    embedding, the TARGET call with the verify model's.  Oracle: the same round with W_draft."""
    block = 16
    W_t = synth.make_head(V, d, 21)
    W_d = (0.8 * W_t.float() + 0.6 * synth.make_head(V, d, 22).float()).to(torch.bfloat16)
    hd, ht = synth.make_hidden(B, K, d, 21, 0.8, 3.0 / (0.02 * np.sqrt(d)))
    vs = fb.VerifyStep(B, K, block, d, V, device=DEV, diag=True, diag_logits=True)
    tok, _, _ = vs(hd.to(DEV), None, W_d.to(DEV), 21, step=2, phase=fb.FEF_PHASE_DRAFT)
    tok, acc, rem = vs(None, ht.to(DEV), W_t.to(DEV), 21, step=2, phase=fb.FEF_PHASE_TARGET)
    torch.cuda.synchronize()
    ref = O.verify_step(synth.to_f64(hd), synth.to_f64(ht), synth.to_f64(W_t), K, block, 21, step=2,
                        return_logits=True, W_draft=synth.to_f64(W_d))
    shared = O.verify_step(synth.to_f64(hd), synth.to_f64(ht), synth.to_f64(W_t), K, block, 21, step=2)
    assert not np.array_equal(ref.draft_tokens, shared.draft_tokens)    # the second head matters
    st = parity.compare(ref, _np(tok), _np(acc), _np(rem), {k: _np(v) for k, v in vs.diag.items()})
    assert st["near_flipped"] <= B // 20


@pytest.mark.parametrize("B,K,d,V,variant", [(1, 8, 512, 3000, fb.FEF_GEMM_AUTO), (2, 8, 512, 3000, fb.FEF_GEMM_AUTO),
                                              (6, 4, 128, 1000, fb.FEF_GEMM_TILED), (40, 4, 64, 700, fb.FEF_GEMM_TILED256),
                                              (24, 4, 64, 700, fb.FEF_GEMM_TILED256)])
def test_split_draft_then_target_call_order(B, K, d, V, variant):
    """The method's own call order: draft laws and draft tokens first, target laws afterwards
    (the verification inputs carry the draft prefix).  The two calls share the workspace; the
    result equals the oracle's and, with the same head kernel, the fused call bit for bit.
    (Above 256 rows the 256 x 256 variant runs its four-wavefront kernel, whose interior tiles sum
    exp over 128 tokens at once and its edge tiles over 64 and 64: a row's partials then depend on
    where its tile lies, and the fused call is held to the oracle instead.)"""
    block = 16
    W = synth.make_head(V, d, 8)
    hd, ht = synth.make_hidden(B, K, d, 8, 0.8, 3.0 / (0.02 * np.sqrt(d)))
    mask = synth.random_mask(B, block, 6, 3)
    Wd, hdd, htd, md = W.to(DEV), hd.to(DEV), ht.to(DEV), torch.as_tensor(mask).to(DEV)
    vs = fb.VerifyStep(B, K, block, d, V, device=DEV, diag=True, diag_logits=True, gemm_variant=variant)
    vs.out_accept_len.fill_(-7)
    tok, _, _ = vs(hdd, None, Wd, 8, step=3, mask_in=md, phase=fb.FEF_PHASE_DRAFT)
    torch.cuda.synchronize()
    drafts = _np(tok).copy()
    assert np.all(_np(vs.out_accept_len) == -7)                # the draft call leaves it alone
    tok, acc, rem = vs(None, htd, Wd, 8, step=3, mask_in=md, phase=fb.FEF_PHASE_TARGET)
    torch.cuda.synchronize()
    ref = O.verify_step(synth.to_f64(hd), synth.to_f64(ht), synth.to_f64(W), K, block, 8, step=3, mask_in=mask,
                        return_logits=True)
    diag = {k: _np(v).copy() for k, v in vs.diag.items()}
    st = parity.compare(ref, _np(tok), _np(acc), _np(rem), diag)
    ok = ref.draft_gap >= parity.TOL_CDF
    assert np.array_equal(drafts[ok], ref.draft_tokens[ok])
    assert st["near_flipped"] <= B // 20
    split = (_np(tok).copy(), _np(acc).copy(), _np(rem).copy(), diag["logits"], diag["alpha"])
    # fused call through the kernel the split calls used
    used = fb.fef_select_gemm(vs._params(), K) if variant != fb.FEF_GEMM_AUTO else None
    p = vs._params(); p.phase = fb.FEF_PHASE_DRAFT
    used = fb.fef_select_gemm(p, K)
    if used != fb.FEF_GEMM_SKINNY or 2 * B * K <= 16:
        vf = fb.VerifyStep(B, K, block, d, V, device=DEV, diag=True, diag_logits=True, gemm_variant=used)
        tok2, acc2, rem2 = vf(hdd, htd, Wd, 8, step=3, mask_in=md)
        torch.cuda.synchronize()
        fused = (_np(tok2), _np(acc2), _np(rem2), _np(vf.diag["logits"]), _np(vf.diag["alpha"]))
        if used == fb.FEF_GEMM_TILED256 and 2 * B * K > 256:
            st2 = parity.compare(ref, fused[0], fused[1], fused[2], {k: _np(v) for k, v in vf.diag.items()})
            assert st2["near_flipped"] <= B // 20
        else:
            for x, y in zip(split, fused):
                assert np.array_equal(x, y)


@pytest.mark.parametrize("case", range(24))
def test_seeded_random_shapes_masks_and_options(case):
    """Seeded draws over what the fixed lists above hold constant: sizes (ragged V, odd multiples of 64
    for d, any K), the head kernel, a random mask with a pass set and confidences, temperature, bases,
    both LowConf scopes, final pass, stochastic re-corruption, greedy."""
    rng = np.random.default_rng(1000 + case)
    variant = [fb.FEF_GEMM_AUTO, fb.FEF_GEMM_TILED, fb.FEF_GEMM_TILED256, fb.FEF_GEMM_STREAM][case % 4]
    K = int(rng.integers(1, 17))
    B = int(rng.integers(1, 128 // (2 * K) + 1)) if variant == fb.FEF_GEMM_STREAM else int(rng.integers(1, 25))
    block = int(rng.integers(K, 41))
    d = 64 * int(rng.integers(1, 10))
    V = int(rng.integers(2, 3000))
    mask = (rng.random((B, block)) < rng.choice([0.2, 0.6, 1.0])).astype(np.uint8)
    mask[0, 0] = 1
    pm = ((1 - mask) * (rng.random((B, block)) < 0.5)).astype(np.uint8)
    conf = (rng.random((B, block)) * (1 - mask)).astype(np.float32)
    greedy = bool(case % 6 == 5)
    ref, out, st = run_case(B, K, block, d, V, seed=200 + case, rho=float(rng.choice([0.5, 0.9, 0.99])),
                            logit_std=float(rng.choice([1.0, 3.0])), variant=variant,
                            temperature=float(rng.choice([0.5, 1.0, 1.3])), step=int(rng.integers(0, 1000)),
                            seq_base=int(rng.integers(0, 1 << 20)), pos_base=int(rng.integers(0, 1 << 16)),
                            n_rm=int(rng.integers(-1, block + 1)), final_pass=bool(rng.random() < 0.2),
                            lowconf_scope=int(case % 2), mask=mask, pass_mask=pm, conf=conf,
                            recorrupt_prob=float(rng.choice([1.0, 0.5])), greedy=greedy)
    print(f"case {case}: B={B} K={K} block={block} d={d} V={V} variant={variant} {st}", flush=True)
    assert st["near_flipped"] <= max(1, B // 10)
    if st["remask_skipped"] == 0 and st["near_margin"] == 0:
        _check_state(ref, out)
