"""Seeded synthetic decode workloads (inputs only).

This module draws the tensors that both the HIP path and the CPU oracle are run on.  It holds
none of the method's arithmetic (no key projection, scoring, selection or attention): it only
draws random tensors, plants "heavy" keys aligned with the query and derives an importance
query that is correlated with the real query, so that the selection has structure to find.

The shapes follow the Llama-class long-context runs the paper measures (Sec. 4.2-4.3: 32 query
heads / 8 KV heads, head_dim 128, 16K-128K context, budgets of a few thousand tokens,
prediction interval 8-16); the public suites and trained predictors behind those runs are not
used, these inputs stand in for them.

The bytes produced are the source of truth: the oracle is fed a host copy of exactly what the
GPU buffers hold, so the stream of random numbers may differ between devices.
"""
from __future__ import annotations

import dataclasses
import math
import zlib
from typing import Dict, Optional

import torch


@dataclasses.dataclass(frozen=True)
class DecodeConfig:
    name: str
    B: int
    Hq: int
    Hkv: int
    D: int
    N: int
    Dimp: int
    k: int
    dtype: str  # "f32" | "bf16"
    heavy_per_kv_head: int  # planted heavy positions per KV head (per step for drifting workloads)
    sink: int = 0
    window: int = 0
    layers: int = 1
    steps: int = 1  # decode steps; the cache grows by one token per step
    P: int = 1  # prediction interval
    radius: int = 0  # neighbour radius on reuse steps
    correlated_q_imp: bool = True  # q_imp = W^T q + noise (False: independent N(0,1))
    zipf_kimp: bool = False  # per-row Zipf(1.2) magnitude scale for the projected keys

    @property
    def g(self) -> int:
        return self.Hq // self.Hkv

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def elt_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def sm_scale(self) -> float:
        return 1.0 / math.sqrt(self.D)

    def scaled(self, **kw) -> "DecodeConfig":
        return dataclasses.replace(self, **kw)

    def algorithmic_bytes(self, total_selected_rows: Optional[int] = None, with_scoring: bool = True) -> int:
        """Projected keys read once per KV head plus gathered K and V rows per query head."""
        if total_selected_rows is None:
            lo = min(self.sink, self.N)
            hi = max(lo, self.N - self.window)
            total_selected_rows = self.B * self.Hq * (lo + min(self.k, hi - lo) + self.N - hi)
        kimp = self.B * self.Hkv * self.N * self.Dimp * self.elt_bytes if with_scoring else 0
        return kimp + total_selected_rows * 2 * self.D * self.elt_bytes


# The five configurations named by the benchmark definition.
C1 = DecodeConfig("C1_tiny_f32", B=1, Hq=8, Hkv=8, D=64, N=1024, Dimp=16, k=128, dtype="f32",
                  heavy_per_kv_head=10, correlated_q_imp=False)
C2 = DecodeConfig("C2_llama3_8b_32k", B=1, Hq=32, Hkv=8, D=128, N=32768, Dimp=32, k=3277, dtype="bf16",
                  heavy_per_kv_head=327)
C3 = DecodeConfig("C3_batched_depth", B=16, Hq=32, Hkv=8, D=128, N=16384, Dimp=32, k=2048, dtype="bf16",
                  heavy_per_kv_head=164, layers=32)
C4 = DecodeConfig("C4_interval_neighbors", B=4, Hq=32, Hkv=8, D=128, N=65536, Dimp=32, k=4096, dtype="bf16",
                  heavy_per_kv_head=65, steps=64, P=8, radius=1)
C5 = DecodeConfig("C5_long_context", B=4, Hq=64, Hkv=8, D=128, N=131072, Dimp=32, k=4096, dtype="bf16",
                  heavy_per_kv_head=655, zipf_kimp=True)
CONFIGS = {c.name: c for c in (C1, C2, C3, C4, C5)}

# Beyond the benchmark definition: the offloaded-cache regime of the paper's efficiency section
# (contexts of 256K and more with K/V in host memory; an 8K-token budget there).
C6 = DecodeConfig("C6_offload_1m", B=1, Hq=32, Hkv=8, D=128, N=1 << 20, Dimp=32, k=8192, dtype="bf16",
                  heavy_per_kv_head=819)
EXTRA_CONFIGS = {c.name: c for c in (C6,)}


def _seed(cfg: DecodeConfig, layer: int, tensor: str, seed: int) -> int:
    return zlib.crc32(f"{cfg.name}/{layer}/{tensor}/{seed}".encode()) & 0x7FFFFFFF


def _randn(shape, cfg, layer, tensor, seed, device) -> torch.Tensor:
    gen = torch.Generator(device=device)
    gen.manual_seed(_seed(cfg, layer, tensor, seed))
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32)


def _rand(shape, cfg, layer, tensor, seed, device) -> torch.Tensor:
    gen = torch.Generator(device=device)
    gen.manual_seed(_seed(cfg, layer, tensor, seed))
    return torch.rand(shape, generator=gen, device=device, dtype=torch.float32)


def make_layer(cfg: DecodeConfig, layer: int = 0, seed: int = 0, device="cpu") -> Dict[str, torch.Tensor]:
    """Draw one layer's decode inputs.

    Returns a dict with
      K, V    [B, Hkv, Ncap, D]   Ncap = N + steps - 1 (the rows a growing cache will reach)
      W       [1, D, Dimp]        one projection matrix per layer, ~ N(0, 1/D)
      q       [steps, B, Hq, D]   real query of each decode step
      q_imp   [steps, B, Hq, Dimp]
      heavy   [B, Hkv, n_heavy] int64  planted base positions (for recall sanity checks)
      kimp_row_scale [B, Hkv, Ncap] fp32 or None  (Zipf magnitude scale, applied by the harness
                                                  to the projected keys after they are computed)
    all in cfg.dtype unless noted.
    """
    dev = torch.device(device)
    B, Hq, Hkv, D, g = cfg.B, cfg.Hq, cfg.Hkv, cfg.D, cfg.g
    steps = cfg.steps
    Ncap = cfg.N + steps - 1
    td = cfg.torch_dtype

    K = _randn((B, Hkv, Ncap, D), cfg, layer, "K", seed, dev)
    V = _randn((B, Hkv, Ncap, D), cfg, layer, "V", seed, dev).to(td)
    W = (_randn((1, D, cfg.Dimp), cfg, layer, "W", seed, dev) / math.sqrt(D)).to(td)
    q = _randn((steps, B, Hq, D), cfg, layer, "q", seed, dev)
    q_unit = q / q.norm(dim=-1, keepdim=True)

    # planted heavy tokens: key <- 3 * q_h / |q_h| + N(0,1), the owning head dealt round-robin
    nh = cfg.heavy_per_kv_head
    gen = torch.Generator(device="cpu")
    gen.manual_seed(_seed(cfg, layer, "heavy", seed))
    heavy = torch.empty((B, Hkv, nh), dtype=torch.int64)
    if steps == 1:
        for b in range(B):
            for h in range(Hkv):
                heavy[b, h] = torch.randperm(cfg.N, generator=gen)[:nh].sort().values
        hv = heavy.to(dev)
        owner = (torch.arange(nh, device=dev) % g).view(1, 1, nh)  # [1,1,nh]
        head = torch.arange(Hkv, device=dev).view(1, Hkv, 1) * g + owner  # [1,Hkv,nh]
        head = head.expand(B, Hkv, nh)
        bidx = torch.arange(B, device=dev).view(B, 1, 1).expand(B, Hkv, nh)
        add = 3.0 * q_unit[0][bidx, head]  # [B,Hkv,nh,D]
        K.scatter_add_(2, hv.unsqueeze(-1).expand(B, Hkv, nh, D), add)
    else:
        # drifting heavy set: streak i occupies rows p_i .. p_i+steps-1; row p_i+t is aligned
        # with the step-t query, so the heavy set moves one position per decode step
        slots = cfg.N // steps
        for b in range(B):
            for h in range(Hkv):
                heavy[b, h] = (torch.randperm(slots, generator=gen)[:nh] * steps).sort().values
        hv = heavy.to(dev)
        owner = (torch.arange(nh, device=dev) % g).view(1, 1, nh)
        head = (torch.arange(Hkv, device=dev).view(1, Hkv, 1) * g + owner).expand(B, Hkv, nh)
        bidx = torch.arange(B, device=dev).view(B, 1, 1).expand(B, Hkv, nh)
        for t in range(steps):
            add = 3.0 * q_unit[t][bidx, head]
            K.scatter_add_(2, (hv + t).unsqueeze(-1).expand(B, Hkv, nh, D), add)
    K = K.to(td)
    q = q.to(td)

    if cfg.correlated_q_imp:
        noise = _randn((steps, B, Hq, cfg.Dimp), cfg, layer, "q_imp", seed, dev)
        q_imp = (torch.einsum("sbhd,dj->sbhj", q.float(), W[0].float()) + 0.1 * noise).to(td)
    else:
        q_imp = _randn((steps, B, Hq, cfg.Dimp), cfg, layer, "q_imp", seed, dev).to(td)

    row_scale = None
    if cfg.zipf_kimp:
        u = _rand((B, Hkv, Ncap), cfg, layer, "zipf", seed, dev).clamp_min(1e-12)
        row_scale = torch.floor(u.pow(-1.0 / 0.2)).clamp(1.0, 65536.0)

    return {"K": K, "V": V, "W": W, "q": q, "q_imp": q_imp, "heavy": heavy, "kimp_row_scale": row_scale}


def apply_kimp_row_scale(Kimp: torch.Tensor, row_scale: Optional[torch.Tensor]) -> torch.Tensor:
    """Multiply each projected-key row by its magnitude scale and round back to the storage
    dtype (input shaping for the sharp-threshold workload; elementwise, in place)."""
    if row_scale is None:
        return Kimp
    n = Kimp.shape[2]
    Kimp.copy_((Kimp.float() * row_scale[:, :, :n].unsqueeze(-1)).to(Kimp.dtype))
    return Kimp
