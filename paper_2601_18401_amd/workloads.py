"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws random tensors and plants structure in them; it contains none of the
method's arithmetic (no scoring, no selection, no softmax), so both the HIP path and the CPU
oracle can be fed from it without sharing code.

Recipe (the same for every run): seed = 20260118 + config number; one torch.Generator on the
generation device; tensors drawn in the order Q, K, V (then, for the needle config, the
direction u, the needle positions and the needle noise).  Values are drawn in fp32 and rounded
once to the storage dtype (round-to-nearest-even); the rounded tensors are the inputs of both
sides.  Large caches are drawn in chunks on the device.
"""
from __future__ import annotations

import dataclasses
import math

import torch

BASE_SEED = 20260118


@dataclasses.dataclass(frozen=True)
class Config:
    name: str
    kind: str          # "prefill" | "decode"
    dtype: str         # "f32" | "bf16"
    L: int
    Hq: int
    Hkv: int
    D: int
    S: int
    topk: int
    input_scale: float = 1.0
    needles: int = 0
    number: int = 0

    @property
    def n_spans(self) -> int:
        return -(-self.L // self.S)

    @property
    def Lq(self) -> int:
        return self.L if self.kind == "prefill" else 1

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def scaled(self, L: int, S: int | None = None, **kw) -> "Config":
        """Same head geometry at a smaller length (parity-test sizes)."""
        return dataclasses.replace(self, L=L, S=S if S is not None else self.S, **kw)


CONFIGS = {
    "C1": Config("C1", "prefill", "f32", 4096, 4, 4, 64, 64, 4, number=1),
    "C2": Config("C2", "prefill", "bf16", 65536, 32, 4, 128, 256, 8, input_scale=1.0 / math.sqrt(128.0), number=2),
    "C3": Config("C3", "decode", "bf16", 1048576, 32, 4, 128, 1024, 16, number=3),
    "C4": Config("C4", "prefill", "bf16", 262144, 32, 4, 128, 512, 8, needles=16, number=4),
    "C5": Config("C5", "decode", "bf16", 10485760, 32, 4, 128, 4096, 16, number=5),
}


def _randn_chunked(shape, gen, device, dtype, scale=1.0, chunk_rows=1 << 20):
    """N(0, scale^2) tensor of `shape` [H, T, D], drawn in fp32 chunks along T and rounded to dtype."""
    H, T, D = shape
    out = torch.empty(shape, dtype=dtype, device=device)
    for h in range(H):
        for t0 in range(0, T, chunk_rows):
            t1 = min(T, t0 + chunk_rows)
            blk = torch.randn((t1 - t0, D), generator=gen, device=device, dtype=torch.float32)
            if scale != 1.0:
                blk.mul_(scale)
            out[h, t0:t1] = blk.to(dtype)
    return out


def generate(cfg: Config, device="cpu", seed: int | None = None, n_queries: int = 1):
    """Returns a dict with Q, K, V (and Qs: the tensor scored against the span keys).

    prefill: Q [Hq, L, D].  decode: Q [n_queries, Hq, 1, D] -- several independent decode
    queries against the same cache, so that timed steps can rotate over different span sets.
    K, V: [Hkv, L, D].  For the needle config also `needle_spans` (sorted int64 tensor).
    """
    seed = BASE_SEED + cfg.number if seed is None else seed
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    dt = cfg.torch_dtype
    out = {}
    if cfg.kind == "prefill":
        Qf = _randn_chunked((cfg.Hq, cfg.L, cfg.D), gen, device, torch.float32, cfg.input_scale)
    else:
        Qf = torch.randn((n_queries, cfg.Hq, 1, cfg.D), generator=gen, device=device,
                         dtype=torch.float32) * cfg.input_scale
    K = _randn_chunked((cfg.Hkv, cfg.L, cfg.D), gen, device, dt, cfg.input_scale)
    V = _randn_chunked((cfg.Hkv, cfg.L, cfg.D), gen, device, dt, cfg.input_scale)
    if cfg.needles:
        # Needle structure: `needles` distinct grid spans (same positions for every kv head) whose
        # keys are 4*u + N(0, 0.1^2); every query of a kv group is g + u with g ~ N(0, I).
        G = cfg.Hq // cfg.Hkv
        u = torch.randn((cfg.Hkv, cfg.D), generator=gen, device=device, dtype=torch.float32)
        pos = torch.randperm(cfg.n_spans, generator=gen, device=device)[: cfg.needles].sort().values
        for j in pos.tolist():
            noise = torch.randn((cfg.Hkv, cfg.S, cfg.D), generator=gen, device=device, dtype=torch.float32)
            K[:, j * cfg.S:(j + 1) * cfg.S] = (4.0 * u[:, None, :] + 0.1 * noise).to(dt)
        Qf = Qf + u.repeat_interleave(G, dim=0)[:, None, :]
        out["needle_spans"] = pos.cpu()
        out["u"] = u
    out["Q"] = Qf.to(dt)
    del Qf
    out["Qs"] = out["Q"]   # the configurations score spans with the attention query tensor
    out["K"] = K
    out["V"] = V
    return out
