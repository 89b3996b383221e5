"""Seeded synthetic inputs for the FeF-DLLM verify step.

This module holds no arithmetic of the method: it only draws random vocabulary heads and
hidden states with the shapes of the paper's workloads (LLaDA-8B: d=4096, V=126464;
Dream-7B: d=3584, V=151936; window k in {4, 8, 16}).  The same tensors feed the HIP path and
the CPU oracle in tests and benchmarks; they stand in for the hidden states a fine-tuned
LLaDA-Instruct would produce on the paper's evaluation prompts, which are not available.

Recipe:
  W[v, :]          ~ N(0, 0.02^2) i.i.d., drawn in fp32 and rounded once to the storage dtype
  h_draft[b, m, :] ~ N(0, sigma_h^2),  sigma_h = logit_std / (0.02 sqrt(d))
  h_target         = rho h_draft + sqrt(1 - rho^2) N(0, sigma_h^2)
so that each logit has standard deviation ~ logit_std and draft and target logits are
correlated with coefficient rho, which moves the acceptance probability sum_v min(p_v, q_v).
"""
import math
from dataclasses import dataclass

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    K: int
    block: int
    gen_len: int
    d: int
    V: int
    dtype: str          # "bf16" | "f32"
    rho: float
    logit_std: float    # 0 -> sigma_h = 1 (the tiny configuration states h ~ N(0,1))
    temperature: float = 1.0
    steps_per_block: int = 64

    @property
    def sigma_h(self):
        return 1.0 if self.logit_std <= 0 else self.logit_std / (0.02 * math.sqrt(self.d))


WORKLOADS = {
    "tiny": Workload("tiny", B=1, K=4, block=8, gen_len=16, d=64, V=32, dtype="f32",
                     rho=0.9, logit_std=0.0),
    "tiny_v8": Workload("tiny_v8", B=1, K=4, block=8, gen_len=16, d=64, V=8, dtype="f32",
                        rho=0.9, logit_std=0.0),
    "llada_b1": Workload("llada_b1", B=1, K=8, block=32, gen_len=256, d=4096, V=126464,
                         dtype="bf16", rho=0.9, logit_std=3.0),
    "llada_k16": Workload("llada_k16", B=1, K=16, block=32, gen_len=256, d=4096, V=126464,
                          dtype="bf16", rho=0.9, logit_std=3.0),
    "llada_b2": Workload("llada_b2", B=2, K=8, block=32, gen_len=256, d=4096, V=126464,
                         dtype="bf16", rho=0.9, logit_std=3.0),
    "llada_b3": Workload("llada_b3", B=3, K=8, block=32, gen_len=256, d=4096, V=126464,
                         dtype="bf16", rho=0.9, logit_std=3.0),
    "llada_b4": Workload("llada_b4", B=4, K=8, block=32, gen_len=256, d=4096, V=126464,
                         dtype="bf16", rho=0.9, logit_std=3.0),
    "llada_b6": Workload("llada_b6", B=6, K=8, block=32, gen_len=256, d=4096, V=126464,
                         dtype="bf16", rho=0.9, logit_std=3.0),
    "llada_b8": Workload("llada_b8", B=8, K=8, block=32, gen_len=256, d=4096, V=126464,
                         dtype="bf16", rho=0.9, logit_std=3.0),
    "llada_b16": Workload("llada_b16", B=16, K=8, block=32, gen_len=256, d=4096, V=126464,
                          dtype="bf16", rho=0.9, logit_std=3.0),
    "llada_b32": Workload("llada_b32", B=32, K=8, block=32, gen_len=256, d=4096, V=126464,
                          dtype="bf16", rho=0.9, logit_std=3.0),
    "dream_b1": Workload("dream_b1", B=1, K=16, block=64, gen_len=512, d=3584, V=151936,
                         dtype="bf16", rho=0.95, logit_std=4.0),
    "dream_b4": Workload("dream_b4", B=4, K=16, block=64, gen_len=512, d=3584, V=151936,
                         dtype="bf16", rho=0.95, logit_std=4.0),
    "dream_b32": Workload("dream_b32", B=32, K=16, block=64, gen_len=512, d=3584, V=151936,
                          dtype="bf16", rho=0.95, logit_std=4.0),
    "sweep_b64": Workload("sweep_b64", B=64, K=16, block=32, gen_len=256, d=4096, V=126464,
                          dtype="bf16", rho=0.9, logit_std=3.0),
}

_TORCH_DTYPE = {"bf16": torch.bfloat16, "f32": torch.float32}


def _gen(seed, *tags):
    g = torch.Generator(device="cpu")
    s = int(seed) & 0xFFFFFFFF
    for t in tags:
        s = (s * 1000003 + int(t) + 0x9E3779B9) & 0x7FFFFFFFFFFFFFFF
    g.manual_seed(s)
    return g


def make_head(V, d, seed, dtype="bf16", std=0.02):
    """Vocabulary head W [V, d] (row v = output embedding of token v), CPU tensor."""
    g = _gen(seed, 101)
    W = torch.randn(V, d, generator=g, dtype=torch.float32)
    W.mul_(std)
    return W.to(_TORCH_DTYPE[dtype])


def make_hidden(B, K, d, seed, rho, sigma_h, dtype="bf16", block_index=0, step=0):
    """Draft and target hidden states [B, K, d] for one speculative round, CPU tensors."""
    g = _gen(seed, 202, block_index, step)
    hd = torch.randn(B, K, d, generator=g, dtype=torch.float32) * sigma_h
    noise = torch.randn(B, K, d, generator=g, dtype=torch.float32) * sigma_h
    ht = rho * hd + math.sqrt(max(0.0, 1.0 - rho * rho)) * noise
    dt = _TORCH_DTYPE[dtype]
    return hd.to(dt), ht.to(dt)


def make_round(wl, seed, block_index=0, step=0, B=None):
    """Hidden states of one round of a named workload (optionally a sub-batch of B rows)."""
    return make_hidden(B or wl.B, wl.K, wl.d, seed, wl.rho, wl.sigma_h, wl.dtype,
                       block_index, step)


def to_f64(t):
    """Exact fp64 numpy copy of a bf16/fp32 torch tensor (both widen exactly)."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def random_mask(B, block, n_unresolved, seed):
    """Block masks with exactly n_unresolved ones per row at random positions."""
    rng = np.random.default_rng(seed)
    m = np.zeros((B, block), np.uint8)
    for b in range(B):
        m[b, rng.choice(block, size=n_unresolved, replace=False)] = 1
    return m
