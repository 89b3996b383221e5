"""A verify step records into a HIP graph (no allocation, no memset, plain kernel launches) and
every replay reproduces the eager result, also with eager work and synchronisations in between."""
import numpy as np
import pytest
import torch

from paper_2605_14305_amd import binding as fb
from paper_2605_14305_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.mark.parametrize("B,K,d,V,variant", [(1, 8, 512, 5000, fb.FEF_GEMM_SKINNY), (6, 4, 128, 1000, fb.FEF_GEMM_TILED),
                                              (40, 4, 64, 700, fb.FEF_GEMM_TILED256),
                                              (6, 8, 256, 3000, fb.FEF_GEMM_STREAM), (3, 8, 512, 900, fb.FEF_GEMM_STREAM),
                                              (3, 8, 512, 9000, fb.FEF_GEMM_ROWSTREAM)])
def test_graph_replays_match_eager(B, K, d, V, variant):
    block = 16
    W = synth.make_head(V, d, 3).to(DEV)
    sigma = 3.0 / (0.02 * np.sqrt(d))
    batches = [tuple(t.to(DEV) for t in synth.make_hidden(B, K, d, 3, 0.8, sigma, "bf16", 0, r)) for r in range(4)]
    vs = fb.VerifyStep(B, K, block, d, V, device=DEV, gemm_variant=variant)
    hd, ht = torch.empty_like(batches[0][0]), torch.empty_like(batches[0][1])
    # eager results first
    want = []
    for a, b in batches:
        hd.copy_(a); ht.copy_(b)
        tok, acc, rem = vs(hd, ht, W, 9, step=4)
        torch.cuda.synchronize()
        want.append((tok.cpu().numpy().copy(), acc.cpu().numpy().copy(), rem.cpu().numpy().copy()))
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        vs(hd, ht, W, 9, step=4)            # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(g):
        vs(hd, ht, W, 9, step=4)
    for rep in range(3):
        for i, (a, b) in enumerate(batches):
            hd.copy_(a); ht.copy_(b)
            vs.out_tokens.fill_(-5)
            g.replay()
            torch.cuda.synchronize()
            got = (vs.out_tokens.cpu().numpy(), vs.out_accept_len.cpu().numpy(), vs.out_remask.cpu().numpy())
            for x, y in zip(got, want[i]):
                assert np.array_equal(x, y), (rep, i)
            # eager work between replays
            tok, acc, rem = vs(batches[(i + 1) % 4][0], batches[(i + 1) % 4][1], W, 9, step=4)
            torch.cuda.synchronize()
            assert np.array_equal(tok.cpu().numpy(), want[(i + 1) % 4][0])
