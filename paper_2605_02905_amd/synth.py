"""Seeded synthetic KV-cache blocks (inputs only; none of the method's arithmetic).

The paper measures on real Llama-3.1-8B / Ministral-8B caches (Sec. 4.1); those
weights and passages are not available, so every test and benchmark input is a
draw from the spiked model the paper itself postulates (Appendix A.1,
Eqs. spiked / separable): S = Z_sig diag(theta) W^T + E, with a low-rank shared
part and a residual with separable (here: diagonal column) covariance, in the
shapes of those models' caches (d = 128, 8 KV heads, 32 / 36 layers).

Both the HIP path and the CPU oracle consume the bytes produced here.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import torch

SEED_BASE = 260502905


@dataclass
class BlockSpec:
    """Recipe of one workload (a list of head-tensors, each `blocks_per_tensor` blocks)."""
    name: str
    n: int                      # tokens per block
    d: int = 128
    n_tensors: int = 1          # (layer, head, K/V) combinations
    blocks_per_tensor: int = 1
    rank_lo: int = 3
    rank_hi: int = 3
    frac_rank0: float = 0.0     # fraction of pure-noise blocks
    strengths: tuple | None = None   # fixed spike strengths in units of sqrt(n) * noise sigma
    strength_mu: float = math.log(4.0)   # lognormal spike strength in BBP units (n d)^{1/4}
    strength_s: float = 0.5
    channel_s: float = 0.7      # lognormal sigma of the per-channel noise scale (0 = white)
    dtype: torch.dtype = torch.float16

    @property
    def n_blocks(self) -> int:
        return self.n_tensors * self.blocks_per_tensor


def config(i: int) -> BlockSpec:
    """The five workloads of the benchmark definition (1-based), and 6: the same layer as 2 cut into the
    128 x 128 blocks of the paper's own experiments (Sec. 3, Tables 1-5), and 7: what one step of a chunked prefill
    hands over, the newest 128 tokens of every layer and head (Sec. 5)."""
    if i == 1:   # single block, fp32, three planted spikes, white noise
        return BlockSpec("cfg1-single-block", n=512, strengths=(6.0, 4.0, 2.5), channel_s=0.0,
                         dtype=torch.float32)
    if i == 2:   # one Llama-3.1-8B-shaped layer: 8 heads x {K,V} x T=32768
        return BlockSpec("cfg2-llama-layer", n=512, n_tensors=16, blocks_per_tensor=64, rank_lo=2, rank_hi=8)
    if i == 3:   # full Llama-3.1-8B-shaped cache: 32 layers
        return BlockSpec("cfg3-llama-cache", n=512, n_tensors=32 * 16, blocks_per_tensor=64, rank_lo=2, rank_hi=8)
    if i == 4:   # one Ministral-8B-shaped layer at T=131072, n=1024 (36 such layers make the cache)
        return BlockSpec("cfg4-ministral-layer", n=1024, n_tensors=16, blocks_per_tensor=128, rank_lo=1, rank_hi=12,
                         frac_rank0=0.10)
    if i == 5:   # keys of 16 sequences x 8 KV heads x T=65536
        return BlockSpec("cfg5-decode-keys", n=512, n_tensors=16 * 8, blocks_per_tensor=128, rank_lo=2, rank_hi=8)
    if i == 6:   # the Llama-shaped layer of config 2 in 128-token blocks
        return BlockSpec("cfg6-llama-layer-n128", n=128, n_tensors=16, blocks_per_tensor=256, rank_lo=1, rank_hi=6)
    if i == 7:   # one 128-token chunk of the whole Llama-3.1-8B-shaped model: 32 layers x {K,V} x 8 heads
        return BlockSpec("cfg7-llama-chunk-n128", n=128, n_tensors=32 * 16, blocks_per_tensor=1, rank_lo=1, rank_hi=6)
    raise ValueError(i)


def _orthonormal_columns(g: torch.Tensor) -> torch.Tensor:
    """Modified Gram-Schmidt on the columns of g [T, d, r] (r small)."""
    cols = []
    for j in range(g.shape[-1]):
        v = g[..., j]
        for c in cols:
            v = v - (v * c).sum(-1, keepdim=True) * c
        cols.append(v / v.norm(dim=-1, keepdim=True))
    return torch.stack(cols, dim=-1)


def make_tensor_blocks(spec: BlockSpec, tensor_index: int, seed: int = SEED_BASE,
                       device: str | torch.device = "cpu", layer: int = 0):
    """Blocks of one head-tensor: returns (blocks [blocks_per_tensor, n, d] of spec.dtype,
    planted_rank [blocks_per_tensor] int64).  Deterministic in (seed, spec.name, layer, tensor_index, device type).
    """
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed((seed * 1000003 + layer * 65537 + tensor_index * 8191 + len(spec.name)) & 0x7FFFFFFFFFFF)
    nb, n, d = spec.blocks_per_tensor, spec.n, spec.d
    rmax = max(spec.rank_hi, 1)
    f32 = dict(device=dev, dtype=torch.float32, generator=gen)
    # per-channel noise scale: a property of the head-tensor, shared by its blocks
    if spec.channel_s > 0:
        c = torch.exp(spec.channel_s * torch.randn(d, **f32))
    else:
        c = torch.ones(d, device=dev)
    rank = torch.randint(spec.rank_lo, spec.rank_hi + 1, (nb,), device=dev, generator=gen)
    if spec.frac_rank0 > 0:
        rank = torch.where(torch.rand(nb, device=dev, generator=gen) < spec.frac_rank0, torch.zeros_like(rank), rank)
    if spec.strengths is not None:
        theta = torch.tensor(spec.strengths, device=dev, dtype=torch.float32).expand(nb, rmax).clone()
    else:
        m = torch.exp(spec.strength_mu + spec.strength_s * torch.randn(nb, rmax, **f32))
        theta = m * (n * d) ** 0.25 / math.sqrt(n)
    theta = theta * (torch.arange(rmax, device=dev)[None, :] < rank[:, None])
    zsig = torch.randn(nb, n, rmax, **f32)
    w = _orthonormal_columns(torch.randn(nb, d, rmax, **f32))
    noise = torch.randn(nb, n, d, **f32) * c
    blocks = torch.baddbmm(noise, zsig * theta[:, None, :], w.transpose(1, 2))
    return blocks.to(spec.dtype), rank


def make_blocks(spec: BlockSpec, seed: int = SEED_BASE, device: str | torch.device = "cpu", layer: int = 0,
                tensors: range | None = None):
    """All (or a range of) head-tensors of a workload, concatenated: ([B, n, d], planted_rank [B])."""
    tensors = range(spec.n_tensors) if tensors is None else tensors
    dev = torch.device(device)
    out = torch.empty(len(tensors) * spec.blocks_per_tensor, spec.n, spec.d, dtype=spec.dtype, device=dev)
    ranks = torch.empty(len(tensors) * spec.blocks_per_tensor, dtype=torch.int64, device=dev)
    for i, t in enumerate(tensors):
        b, r = make_tensor_blocks(spec, t, seed, dev, layer)
        out[i * spec.blocks_per_tensor:(i + 1) * spec.blocks_per_tensor] = b
        ranks[i * spec.blocks_per_tensor:(i + 1) * spec.blocks_per_tensor] = r
    return out, ranks


def make_queries(n_seq: int, n_q_heads: int, d: int = 128, seed: int = SEED_BASE + 7,
                 device: str | torch.device = "cpu", scale: float | None = None, dtype=torch.float16):
    """Decode queries iid N(0, 1/d) (or N(0, scale^2)), [n_seq, n_q_heads, d]."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    s = (1.0 / math.sqrt(d)) if scale is None else scale
    return (torch.randn(n_seq, n_q_heads, d, device=dev, dtype=torch.float32, generator=gen) * s).to(dtype)
