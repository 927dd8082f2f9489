"""Seeded synthetic inputs for the ReST-KV eviction path.

This module only draws random tensors of the shapes and value structure of the
benchmark configurations; it holds none of the method's arithmetic and is the
one piece shared by the HIP tests, the CPU oracle tests and the benchmark.  The
paper evaluates on long-context suites with real model weights; neither is
available here, so these tensors stand in for them by shape only.

Every tensor is a pure function of (config, layer, seed, device type): the same
call gives the same values on the same device type.  Large configurations are
generated directly on the GPU and the oracle receives copies of those bytes.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seq_len: int
    window: int
    budget: int
    dtype: str            # "f32" | "bf16"
    d_model: int          # width D of the output projection [Hq*d, D]
    alpha: float          # EMA factor on the newest query (decay = 1 - alpha)
    base_window: int      # spatial kernel k
    beta: float           # adaptive-window scaling factor
    structure: str        # "plain" | "sinks" | "lowrank" | "drift"
    seed: int

    def __post_init__(self):
        # The library's parameter block carries alpha and beta as FP32.  The workload holds exactly
        # those values, so that every consumer sees the same numbers (1 - alpha differs by 1.3e-5
        # between 0.999 and its nearest FP32 neighbour).
        for name in ("alpha", "beta"):
            object.__setattr__(self, name, float(torch.tensor(getattr(self, name), dtype=torch.float32).item()))

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def prefix(self) -> int:
        return self.seq_len - self.window

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS: Dict[str, Workload] = {
    # 1 layer, 2 KV heads x 2 query heads, fp32, decay 0.9 -> alpha 0.1
    "tiny": Workload("tiny", 1, 4, 2, 64, 1024, 32, 128, "f32", 128, 0.1, 5, 2000.0, "plain", 0x5EED + 1),
    # single Llama-3-8B-like layer, 4 planted heavy keys per KV head (x8)
    "llama_8k": Workload("llama_8k", 1, 32, 8, 128, 8192, 32, 512, "bf16", 4096, 0.3, 5, 2000.0, "sinks", 0x5EED + 2),
    # 32 layers, rank-16 shared key/query structure per KV head
    "lowrank_32k": Workload("lowrank_32k", 32, 32, 8, 128, 32768, 64, 1024, "bf16", 4096, 0.3, 5, 2000.0, "lowrank", 0x5EED + 3),
    # 32 layers at 128k, keys with a slowly drifting mean (random walk, sigma 0.01)
    "drift_128k": Workload("drift_128k", 32, 32, 8, 128, 131072, 64, 2048, "bf16", 4096, 0.3, 5, 2000.0, "drift", 0x5EED + 4),
    # 80 layers, 64 query heads over 8 KV heads
    "gqa8_128k": Workload("gqa8_128k", 80, 64, 8, 128, 131072, 64, 1024, "bf16", 8192, 0.3, 5, 2000.0, "plain", 0x5EED + 5),
    # Decode-time re-eviction (App. B): a cache held at budget B = 2048 has grown by M = 64 generated
    # tokens; their queries are the observation window and the cache goes back to B.  Not one of the
    # five benchmark configurations: the small-L regime of the same path.
    "decode_reevict": Workload("decode_reevict", 32, 32, 8, 128, 2048 + 64, 64, 2048, "bf16", 4096, 0.3, 5, 2000.0, "drift", 0x5EED + 6),
}


def torch_dtype(w: Workload) -> torch.dtype:
    return torch.float32 if w.dtype == "f32" else torch.bfloat16


def _gen(w: Workload, layer: int, stream: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((w.seed * 1_000_003 + layer * 1009 + stream) & 0x7FFF_FFFF_FFFF)
    return g


def make_qkv(w: Workload, layer: int = 0, device="cpu"):
    """q [Hq,W,d], k,v [Hkv,L,d] in the workload's dtype (post-RoPE by assumption)."""
    dev = torch.device(device)
    Hq, Hkv, d, L, W = w.n_q_heads, w.n_kv_heads, w.head_dim, w.seq_len, w.window
    G = w.group
    f32 = torch.float32
    q = torch.randn((Hq, W, d), generator=_gen(w, layer, 0, dev), device=dev, dtype=f32)
    k = torch.randn((Hkv, L, d), generator=_gen(w, layer, 1, dev), device=dev, dtype=f32)
    v = torch.randn((Hkv, L, d), generator=_gen(w, layer, 2, dev), device=dev, dtype=f32)
    if w.structure == "sinks":
        # position 0 and three seeded prefix positions per KV head carry keys scaled x8
        g = _gen(w, layer, 3, torch.device("cpu"))
        for h in range(Hkv):
            pos = torch.randint(1, max(w.prefix, 2), (3,), generator=g).tolist()   # (a one-token prefix: position 1 is in the window)
            for p in [0] + pos:
                k[h, p, :] *= 8.0
    elif w.structure == "lowrank":
        r = 16
        g = _gen(w, layer, 3, dev)
        F = torch.randn((Hkv, r, d), generator=g, device=dev, dtype=f32) * (1.0 / r) ** 0.5
        ck = torch.randn((Hkv, L, r), generator=g, device=dev, dtype=f32)
        cq = torch.randn((Hq, W, r), generator=g, device=dev, dtype=f32)
        k += torch.bmm(ck, F)
        q += torch.bmm(cq, F.repeat_interleave(G, dim=0))
    elif w.structure == "drift":
        g = _gen(w, layer, 3, dev)
        for h in range(Hkv):       # per head to bound the temporary; scan along the fast axis
            step = torch.randn((d, L), generator=g, device=dev, dtype=f32) * 0.01
            k[h] += torch.cumsum(step, dim=1).t()
    elif w.structure != "plain":
        raise ValueError(w.structure)
    dt = torch_dtype(w)
    return q.to(dt), k.to(dt), v.to(dt)


def make_wo(w: Workload, layer: int = 0, device="cpu") -> torch.Tensor:
    """Output projection [Hq*d, D] fp32, entries N(0, 1/D), in the z @ W_O orientation."""
    dev = torch.device(device)
    g = _gen(w, layer, 7, dev)
    wo = torch.randn((w.n_q_heads * w.head_dim, w.d_model), generator=g, device=dev,
                     dtype=torch.float32)
    return wo * (1.0 / w.d_model) ** 0.5


def small_case(name: str = "small", *, Hq=4, Hkv=2, d=64, L=300, W=8, B=40, dtype="f32",
               D: Optional[int] = None, alpha=0.3, k=5, beta=2000.0, structure="plain",
               seed=1234) -> Workload:
    """Ad-hoc workload for tests (ragged sizes, several tiles, odd windows ...)."""
    return Workload(name, 1, Hq, Hkv, d, L, W, B, dtype, D if D is not None else Hq * d // 2,
                    alpha, k, beta, structure, seed)
