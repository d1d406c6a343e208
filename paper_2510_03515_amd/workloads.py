"""Seeded synthetic workloads standing in for RAPID's MBPP+/MATH/MiniF2F mini-batches.

Input generation only: no part of the estimator (log-softmax, ratios, advantages, gradients)
lives here.  Both the HIP path and the CPU oracle consume exactly the tensors made here, after
rounding to the storage dtype, so the two see the same bits.

Recipe (draw order: lengths, hidden, W, W_old perturbation, tokens, rewards):
  lengths  L_n ~ UniformInt[lo, hi]; mask[n,t] = t < L_n; T = hi
  hidden   N(0,1) rows divided by their RMS (padded rows filled the same way), then rounded
  W        N(0, 0.02^2), logical [d,V]; W_old = W + N(0, sigma^2); both rounded after the add
  tokens   y ~ softmax(h W_old) by the Gumbel-max trick, row-chunked; padded positions get id 0
  rewards  Bernoulli(p) or U[0,1]; optionally group 0 forced all-0 and group 1 all-1
  groups   group_ids[n] = n // G
Shapes follow the Qwen2.5-0.5B/1.5B/3B LM heads (d = 896/1536/2048, V = 151936) and the paper's
max completion length of 2048 tokens (Appendix A).
"""
from __future__ import annotations

import dataclasses
import math

import torch


@dataclasses.dataclass(frozen=True)
class WorkloadSpec:
    name: str
    dtype: str            # "f32" | "bf16"
    d: int
    V: int
    prompts: int
    G: int
    len_lo: int
    len_hi: int
    sigma: float          # std of W_old - W
    reward: str           # "bernoulli" | "uniform"
    reward_p: float = 0.4
    force_edge_groups: bool = False
    tokens_from: str = "old"   # "old": y ~ softmax(h W_old); "cur": y ~ softmax(h W)
    fwd_only: bool = False

    @property
    def N(self):
        return self.prompts * self.G

    @property
    def T(self):
        return self.len_hi


CONFIGS = [
    WorkloadSpec("cfg0_tiny_f32", "f32", 64, 1000, 8, 4, 8, 32, 0.01, "bernoulli", 0.4),
    WorkloadSpec("cfg1_qwen0.5b", "bf16", 896, 151936, 16, 8, 128, 1024, 0.005, "bernoulli", 0.4),
    WorkloadSpec("cfg2_qwen1.5b", "bf16", 1536, 151936, 32, 8, 256, 2048, 0.01, "bernoulli", 0.3,
                 force_edge_groups=True),
    WorkloadSpec("cfg3_qwen3b", "bf16", 2048, 151936, 16, 16, 512, 4096, 0.02, "uniform"),
    WorkloadSpec("cfg4_behaviour_fwd", "bf16", 1536, 151936, 512, 1, 1024, 1024, 0.0, "bernoulli",
                 0.4, tokens_from="cur", fwd_only=True),
    # one 65536-row backward chunk of the Qwen2.5-1.5B shape (no padding): every kernel of the path
    # launches exactly once, which keeps hardware-counter passes short
    WorkloadSpec("cfg2_one_chunk", "bf16", 1536, 151936, 4, 8, 2048, 2048, 0.01, "bernoulli", 0.3),
]


def calibrated(spec: WorkloadSpec) -> WorkloadSpec:
    """Same shapes, seed and rewards with sigma' = sqrt(0.5 / (T d)), so that the generation-level
    log ratio stays O(1) and a few per cent of the weights clip (the regime of the paper's
    staleness table and clip-proportion figure)."""
    return dataclasses.replace(spec, name=spec.name + "_calibrated",
                               sigma=math.sqrt(0.5 / (spec.T * spec.d)))


def _torch_dtype(name):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def make_workload(spec: WorkloadSpec, seed: int = 0, device: str = "cpu", row_chunk: int = 4096):
    """Returns a dict of tensors on `device`:
    hidden [N,T,d] dtype, W [d,V] dtype, W_old [d,V] dtype, tokens [N,T] int32, mask [N,T] uint8,
    rewards [N] f32, group_ids [N] int32, lengths [N] int64; plus K and the spec."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    dt = _torch_dtype(spec.dtype)
    N, T, d, V = spec.N, spec.T, spec.d, spec.V

    lengths = torch.randint(spec.len_lo, spec.len_hi + 1, (N,), generator=gen, device=dev)
    mask = (torch.arange(T, device=dev)[None, :] < lengths[:, None]).to(torch.uint8)

    hidden = torch.empty((N, T, d), dtype=dt, device=dev)
    for n0 in range(0, N, 8):
        h = torch.randn((min(8, N - n0), T, d), generator=gen, device=dev, dtype=torch.float32)
        h = h / h.pow(2).mean(dim=-1, keepdim=True).sqrt()
        hidden[n0:n0 + h.shape[0]] = h.to(dt)

    W32 = torch.randn((d, V), generator=gen, device=dev, dtype=torch.float32) * 0.02
    W = W32.to(dt)
    if spec.sigma > 0:
        W_old = (W32 + torch.randn((d, V), generator=gen, device=dev, dtype=torch.float32)
                 * spec.sigma).to(dt)
    else:
        W_old = W.clone()
    del W32

    W_samp = W_old if spec.tokens_from == "old" else W
    tokens = torch.zeros((N, T), dtype=torch.int32, device=dev)
    flat_h = hidden.view(N * T, d)
    valid = torch.nonzero(mask.view(-1), as_tuple=False).view(-1)
    for s in range(0, valid.numel(), row_chunk):
        idx = valid[s:s + row_chunk]
        if dev.type == "cuda":
            z = (flat_h[idx] @ W_samp).float()
        else:
            z = flat_h[idx].float() @ W_samp.float()
        u = torch.rand(z.shape, generator=gen, device=dev, dtype=torch.float32)
        z = z - torch.log(-torch.log(u.clamp_min(1e-30)).clamp_min(1e-30))
        tokens.view(-1)[idx] = z.argmax(dim=1).to(torch.int32)
        del z, u

    if spec.reward == "bernoulli":
        rewards = (torch.rand((N,), generator=gen, device=dev) < spec.reward_p).float()
    else:
        rewards = torch.rand((N,), generator=gen, device=dev).float()
    group_ids = (torch.arange(N, device=dev) // spec.G).to(torch.int32)
    if spec.force_edge_groups and spec.prompts >= 2:
        rewards[group_ids == 0] = 0.0
        rewards[group_ids == 1] = 1.0

    return dict(spec=spec, hidden=hidden, W=W, W_old=W_old, tokens=tokens, mask=mask,
                rewards=rewards, group_ids=group_ids, lengths=lengths, K=spec.prompts)


def small_spec(name="small", dtype="bf16", d=128, V=1000, prompts=4, G=4, len_lo=3, len_hi=40,
               sigma=0.01, reward="bernoulli", **kw):
    """Reduced-size spec with the same recipe, for parity tests the oracle finishes in seconds."""
    return WorkloadSpec(name, dtype, d, V, prompts, G, len_lo, len_hi, sigma, reward, **kw)
