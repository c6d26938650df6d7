"""Seeded synthetic workloads for the LCKV decode step.

This module only draws random numbers and lengths and describes shapes.  It
holds none of the method's arithmetic and no cache layout: both the GPU path's
tests and the CPU oracle's tests take their inputs from here.

The shapes stand in for the generation workloads of the paper's throughput
study (Section 3.1, Table 1; model shapes from the appendix table "Model
configurations"): cost depends only on shapes and lengths, so Q, K and V are
i.i.d. normal draws and the lengths are fixed or uniform.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Optional, Tuple

import numpy as np
import torch

PAGE = 16  # tokens per page of the paged cache layout

BASE_SEED = 240510637000


def sandwich_mask(L: int, w: int) -> np.ndarray:
    """Warmup layers in the sandwich placement (Section 2.1): bottom w/2 and top w/2 layers.

    An odd w puts the extra layer at the bottom.
    """
    if not 0 <= w <= L:
        raise ValueError("need 0 <= w <= L")
    m = np.zeros(L, np.uint8)
    top = w // 2
    bottom = w - top
    m[:bottom] = 1
    if top:
        m[L - top:] = 1
    return m


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str            # "bf16" | "f32"
    L: int
    w: int                # number of warmup layers, sandwich placement unless `warm` is given
    Hq: int
    Hkv: int
    D: int
    B: int
    T: int                # cached length before the step (uniform) or the maximum when ragged
    T_min: Optional[int] = None   # ragged: lengths uniform in [T_min, T], both ends included
    paged: bool = False
    sigma: float = 0.5
    seed: int = BASE_SEED
    warm: Optional[Tuple[int, ...]] = None

    @property
    def warmup_mask(self) -> np.ndarray:
        if self.warm is not None:
            m = np.zeros(self.L, np.uint8)
            m[list(self.warm)] = 1
            return m
        return sandwich_mask(self.L, self.w)

    @property
    def torch_dtype(self):
        return {"bf16": torch.bfloat16, "f32": torch.float32}[self.dtype]

    @property
    def elem_bytes(self) -> int:
        return {"bf16": 2, "f32": 4}[self.dtype]

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


# The five named workloads.  C3 is the headline.
C1 = Workload("C1-tiny-f32", "f32", L=4, w=1, Hq=4, Hkv=4, D=64, B=2, T=128, sigma=1.0,
              seed=BASE_SEED + 1, warm=(0,))
C2 = Workload("C2-tinyllama-1.1b", "bf16", L=22, w=2, Hq=32, Hkv=4, D=64, B=64, T=2048, seed=BASE_SEED + 2)
C3 = Workload("C3-llama-7b", "bf16", L=32, w=2, Hq=32, Hkv=32, D=128, B=128, T=4096, seed=BASE_SEED + 3)
C4 = Workload("C4-llama-7b-ragged-paged", "bf16", L=32, w=2, Hq=32, Hkv=32, D=128, B=256, T=8192, T_min=256,
              paged=True, seed=BASE_SEED + 4)
C5 = Workload("C5-13b-shape-long", "bf16", L=40, w=10, Hq=40, Hkv=40, D=128, B=16, T=32768, seed=BASE_SEED + 5)
WORKLOADS = {"C1": C1, "C2": C2, "C3": C3, "C4": C4, "C5": C5}


def seq_lens(wl: Workload) -> np.ndarray:
    """Tokens cached per sequence before the step (int32 [B])."""
    if wl.T_min is None:
        return np.full(wl.B, wl.T, np.int32)
    rng = np.random.Generator(np.random.Philox(key=wl.seed + 101))
    return rng.integers(wl.T_min, wl.T + 1, size=wl.B, dtype=np.int32)


def block_table(wl: Workload, lens: np.ndarray, extra_tokens: int = 1):
    """Paged workloads: (table int32 [B][max_blocks], num_blocks).

    Sequence b gets ceil((lens[b] + extra_tokens) / PAGE) blocks; physical block ids are a seeded random
    permutation of [0, num_blocks).  Unused table entries are -1.
    """
    need = (lens.astype(np.int64) + extra_tokens + PAGE - 1) // PAGE
    num_blocks = int(need.sum())
    rng = np.random.Generator(np.random.Philox(key=wl.seed + 202))
    perm = rng.permutation(num_blocks).astype(np.int32)
    max_blocks = int(need.max())
    table = np.full((wl.B, max_blocks), -1, np.int32)
    at = 0
    for b in range(wl.B):
        table[b, : need[b]] = perm[at: at + need[b]]
        at += need[b]
    return table, num_blocks


def _normal(shape, sigma: float, dtype, seed: int, device="cpu") -> torch.Tensor:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    t = torch.empty(shape, dtype=torch.float32, device=device)
    t.normal_(0.0, sigma, generator=g)
    return t.to(dtype)  # round-to-nearest-even for bf16


def step_inputs(wl: Workload, n_slots: int, device="cpu", step: int = 0):
    """(q [L][B][Hq][D], k_new [n_slots][B][Hkv][D], v_new likewise) in the workload's dtype."""
    s = wl.seed * 7 + 1000 * step
    q = _normal((wl.L, wl.B, wl.Hq, wl.D), wl.sigma, wl.torch_dtype, s + 1, device)
    k = _normal((n_slots, wl.B, wl.Hkv, wl.D), wl.sigma, wl.torch_dtype, s + 2, device)
    v = _normal((n_slots, wl.B, wl.Hkv, wl.D), wl.sigma, wl.torch_dtype, s + 3, device)
    return q, k, v


def logical_cache(wl: Workload, n_slots: int, T_cap: int):
    """Dense logical caches K, V of shape [n_slots][B][T_cap][Hkv][D] on the CPU (small workloads only).

    Every position is filled, also those beyond a sequence's length: what lies there must not matter.
    """
    shape = (n_slots, wl.B, T_cap, wl.Hkv, wl.D)
    K = _normal(shape, wl.sigma, wl.torch_dtype, wl.seed * 7 + 11)
    V = _normal(shape, wl.sigma, wl.torch_dtype, wl.seed * 7 + 12)
    return K, V


def fill_normal_(t: torch.Tensor, sigma: float, seed: int, chunk_elems: int = 1 << 28) -> torch.Tensor:
    """Fill a (large, device) tensor in place with sigma * N(0,1) draws, chunk by chunk."""
    flat = t.view(-1)
    g = torch.Generator(device=t.device)
    g.manual_seed(seed)
    for at in range(0, flat.numel(), chunk_elems):
        part = flat[at: at + chunk_elems]
        tmp = torch.empty(part.shape, dtype=torch.float32, device=t.device)
        tmp.normal_(0.0, sigma, generator=g)
        part.copy_(tmp)
    return t


def sample_units(wl: Workload, lens: np.ndarray, n: int, must_layers=()):
    """Seeded sample of (layer, b, query head) triples; always holds the corners named in the test plan:
    first/last layer, the layers in `must_layers`, b = 0 and B-1, the shortest and the longest sequence."""
    rng = np.random.Generator(np.random.Philox(key=wl.seed + 303))
    layers = sorted(set([0, wl.L - 1]) | set(int(x) for x in must_layers))
    bs = sorted(set([0, wl.B - 1, int(np.argmin(lens)), int(np.argmax(lens))]))
    units = []
    for l in layers:
        for b in bs:
            units.append((l, b, int(rng.integers(0, wl.Hq))))
    while len(units) < n:
        units.append((int(rng.integers(0, wl.L)), int(rng.integers(0, wl.B)), int(rng.integers(0, wl.Hq))))
    return units[: max(n, len(layers) * len(bs))]
