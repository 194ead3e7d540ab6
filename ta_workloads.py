"""Seeded synthetic inputs for decode attention.

This module only draws random tensors of the stated shapes and distributions.
It holds none of the method's arithmetic and imports neither the HIP package
nor the oracle; tests and the benchmark hand the same tensors to both.

Recipes (config index k uses seed 20240804 + k):
  0 tiny      B=1 Hq=Hkv=1 d=64 N=4096 fp32, N(0,1), scale 1/sqrt(d); 16 chunks of 256
  1 llama128k B=1 Hq=32 Hkv=8 d=128 N=131072 bf16, N(0,1), scale 1/sqrt(128)
  2 ragged    B=16 Hq=32 Hkv=8 d=128 bf16, KV padded to 65536,
              valid_len[b] uniform on {8192..65536}
  3 million   B=1 Hq=32 Hkv=8 d=128 N=1048576 bf16, N(0,1); for every (b, kv head)
              floor(0.01 N) distinct rows of K (seeded permutation) get one scalar
              offset ~ Normal(0, std 2) added to all d components in fp32 before
              rounding to bf16 (peaked attention, same byte count)
  4 combine   B=4 Hq=64 Hkv=8 d=128 N=262144 bf16, N(0,1); chunk bounds = 0, P-1
              distinct cut points uniform on {1..N-1} sorted, N (P=64), shared
              by every (b, h)
  5 shard     the paper's own micro-benchmark shard: one device's share of its 16-head,
              d=128, bf16 attention block (Section 6.1): B=1 Hq=Hkv=16, N=80000
              (640 000 tokens over 8 GPUs, Section 6.3) or N=40000 (5.12 M over 128),
              N(0,1) with q multiplied by 1/sqrt(128), scale 1 as in the paper
Every generator takes size overrides so tests can run the same recipe small.
"""
from dataclasses import dataclass, field
from typing import Optional

import torch

BASE_SEED = 20240804


@dataclass
class Workload:
    name: str
    q: torch.Tensor                      # [B,Hq,d]
    K: torch.Tensor                      # [B,Hkv,N,d]
    V: torch.Tensor                      # [B,Hkv,N,d]
    scale: float
    valid_len: Optional[torch.Tensor] = None     # int32 [B] or None
    chunk_bounds: Optional[torch.Tensor] = None  # int64 [P+1] or None
    meta: dict = field(default_factory=dict)

    @property
    def shape(self):
        B, Hq, d = self.q.shape[0], self.q.shape[-2], self.q.shape[-1]
        _, Hkv, N, _ = self.K.shape
        return B, Hq, Hkv, d, N

    def kv_bytes(self) -> int:
        """Bytes of the valid K and V rows (each read once by the method)."""
        B, Hq, Hkv, d, N = self.shape
        rows = int(self.valid_len.sum().item()) if self.valid_len is not None else B * N
        return 2 * rows * Hkv * d * self.K.element_size()

    def to(self, device):
        mv = lambda t: None if t is None else t.to(device)
        return Workload(self.name, mv(self.q), mv(self.K), mv(self.V), self.scale,
                        mv(self.valid_len), mv(self.chunk_bounds), dict(self.meta))


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _randn(shape, dtype, g, device):
    # drawn in fp32 and rounded once (round-to-nearest-even) to the storage type
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32).to(dtype)


def _randn_big(shape, dtype, g, device):
    """randn for multi-GiB tensors: filled slice by slice to bound the fp32 temporary."""
    out = torch.empty(shape, dtype=dtype, device=device)
    flat = out.view(-1, shape[-2], shape[-1])
    for i in range(flat.shape[0]):
        flat[i] = torch.randn(flat.shape[1:], generator=g, device=device, dtype=torch.float32).to(dtype)
    return out


def make_qkv(B, Hq, Hkv, d, N, dtype, seed, device="cpu", scale=None, q_mult=1.0, name="custom"):
    """q, K, V ~ N(0,1) i.i.d.; q optionally multiplied by q_mult before rounding."""
    g = _gen(seed, device)
    q = (torch.randn((B, Hq, d), generator=g, device=device, dtype=torch.float32) * q_mult).to(dtype)
    K = _randn_big((B, Hkv, N, d), dtype, g, device)
    V = _randn_big((B, Hkv, N, d), dtype, g, device)
    return Workload(name, q, K, V, float(scale if scale is not None else d ** -0.5),
                    meta=dict(seed=seed, q_mult=q_mult))


def make_multi(B, Sq, Hq, Hkv, d, N, dtype, seed, device="cpu", scale=None, name="multi"):
    """Like make_qkv with Sq query tokens per sequence: q [B,Sq,Hq,d]."""
    g = _gen(seed, device)
    q = torch.randn((B, Sq, Hq, d), generator=g, device=device, dtype=torch.float32).to(dtype)
    K = _randn_big((B, Hkv, N, d), dtype, g, device)
    V = _randn_big((B, Hkv, N, d), dtype, g, device)
    return Workload(name, q, K, V, float(scale if scale is not None else d ** -0.5), meta=dict(seed=seed, Sq=Sq))


def tiny(N=4096, q_mult=1.0, device="cpu", d=64, dtype=torch.float32):
    w = make_qkv(1, 1, 1, d, N, dtype, BASE_SEED + 0, device, q_mult=q_mult, name="tiny")
    w.meta["chunk"] = 256
    return w


def llama128k(N=131072, device="cpu", B=1, Hq=32, Hkv=8, d=128, seed_offset=0):
    return make_qkv(B, Hq, Hkv, d, N, torch.bfloat16, BASE_SEED + 1 + 1000 * seed_offset, device,
                    name="llama128k")


def ragged(B=16, N=65536, min_len=8192, device="cpu", Hq=32, Hkv=8, d=128):
    w = make_qkv(B, Hq, Hkv, d, N, torch.bfloat16, BASE_SEED + 2, device, name="ragged")
    g = _gen(BASE_SEED + 2 + 500, "cpu")
    w.valid_len = torch.randint(min_len, N + 1, (B,), generator=g, dtype=torch.int32).to(device)
    return w


def million(N=1048576, device="cpu", B=1, Hq=32, Hkv=8, d=128, frac=0.01, offset_std=2.0):
    seed = BASE_SEED + 3
    g = _gen(seed, device)
    q = torch.randn((B, Hq, d), generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
    K = torch.empty((B, Hkv, N, d), dtype=torch.bfloat16, device=device)
    n_off = int(frac * N)
    for b in range(B):
        for h in range(Hkv):
            k32 = torch.randn((N, d), generator=g, device=device, dtype=torch.float32)
            rows = torch.randperm(N, generator=g, device=device)[:n_off]
            delta = torch.randn((n_off, 1), generator=g, device=device, dtype=torch.float32) * offset_std
            k32[rows] += delta
            K[b, h] = k32.to(torch.bfloat16)
    V = _randn_big((B, Hkv, N, d), torch.bfloat16, g, device)
    return Workload("million", q, K, V, float(d ** -0.5),
                    meta=dict(seed=seed, frac=frac, offset_std=offset_std))


def combine_stress(N=262144, P=64, device="cpu", B=4, Hq=64, Hkv=8, d=128):
    w = make_qkv(B, Hq, Hkv, d, N, torch.bfloat16, BASE_SEED + 4, device, name="combine")
    w.chunk_bounds = random_bounds(N, P, BASE_SEED + 4 + 500).to(device)
    return w


def paper_shard(N=80000, device="cpu"):
    w = make_qkv(1, 16, 16, 128, N, torch.bfloat16, BASE_SEED + 5, device, scale=1.0, name=f"shard{N}")
    # with scale 1 and unit-variance q the scores have std ~11 and all weight lands on one key;
    # q carries the 1/sqrt(d) instead
    w.q = (w.q.float() * (128 ** -0.5)).to(torch.bfloat16)
    return w


def random_bounds(N, P, seed):
    """0, then P-1 distinct cut points uniform on {1..N-1} (sorted), then N."""
    if P - 1 > N - 1:
        raise ValueError("more cut points than positions")
    g = _gen(seed, "cpu")
    cuts = (torch.randperm(N - 1, generator=g)[:P - 1] + 1).sort().values.to(torch.int64)
    return torch.cat([torch.zeros(1, dtype=torch.int64), cuts, torch.tensor([N], dtype=torch.int64)])


def equal_bounds(N, P):
    """P contiguous chunks of ceil(N/P) keys (the last ones may be short or empty)."""
    t = -(-N // P)
    return torch.tensor([min(j * t, N) for j in range(P + 1)], dtype=torch.int64)
