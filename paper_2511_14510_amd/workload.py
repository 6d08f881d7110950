"""Seeded synthetic inputs for the QSAC decode step.

This module holds none of the method's arithmetic: it only draws the random
tensors that both the HIP path and the test oracle consume (the same bits go to
both).  The shapes follow the models the paper evaluates (Section 7.1:
Llama3-8B, 32 query / 8 KV heads; Qwen2.5-14B, 40 query / 8 KV heads; 128
16-bit elements per K/V vector, Section 6.2); the values are synthetic and
stand in for the paper's benchmark runs, which need model weights and datasets.

Recipe
  K, V   i.i.d. N(0,1); per KV head four distinct "outlier" channels (the same
         for K and V of that head, shared across the batch) are multiplied by
         8 before rounding once to fp16 / bf16.
  q_t    q_0 = normalize(e_0); q_t = normalize(rho q_{t-1} + sqrt(1-rho^2) e_t)
         with e_t ~ N(0, I/D), so cos(q_t, q_{t-1}) is rho up to a jitter of a
         few hundredths; every query head runs its own chain (the low-similarity
         workload draws one rho per KV head from U[0.3, 0.99], shared by the
         query heads of the group).  ``exact=True``
         orthogonalises e_t against q_{t-1} and normalises it, which makes the
         cosine exactly rho before rounding.  ``q_norm`` rescales the emitted
         queries (the gate and the ranking do not depend on it; a large norm
         makes the softmax peaked).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch

DEFAULT_SEED = 20251114
N_OUTLIER_CHANNELS = 4
OUTLIER_SCALE = 8.0

TORCH_DTYPES = {"f16": torch.float16, "bf16": torch.bfloat16}
DTYPE_CODES = {"f16": 0, "bf16": 1}


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    Hq: int
    Hkv: int
    N: int
    k: int
    dtype: str
    steps: int
    tau: float = 0.9
    rho: float = 0.95          # scalar; rho_range overrides it with one value per KV head
    rho_range: tuple | None = None
    host_k: bool = False       # fill source of K rows lives in pinned host memory
    host_v: bool = False       # fill source of V rows lives in pinned host memory
    D: int = 128
    seed: int = DEFAULT_SEED

    @property
    def P(self):
        return self.B * self.Hkv

    @property
    def G(self):
        return self.Hq // self.Hkv


CONFIGS = {
    "tiny": Workload("tiny", 1, 8, 2, 4096, 256, "f16", 64),
    "llama3_8b_32k": Workload("llama3_8b_32k", 8, 32, 8, 32768, 2048, "bf16", 256),
    "qwen25_14b_128k_offload": Workload("qwen25_14b_128k_offload", 4, 40, 8, 131072, 2048, "bf16", 128,
                                        host_k=True, host_v=True),
    "long_1m": Workload("long_1m", 1, 32, 8, 1048576, 4096, "bf16", 64, host_v=True),
    "low_sim_stress": Workload("low_sim_stress", 32, 32, 8, 65536, 2048, "bf16", 128,
                               rho_range=(0.3, 0.99), host_k=True, host_v=True),
}


def outlier_channels(Hkv: int, D: int, seed: int) -> np.ndarray:
    """[Hkv, 4] distinct channel numbers per KV head."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 0xC4A7]))
    return np.stack([rng.choice(D, size=N_OUTLIER_CHANNELS, replace=False) for _ in range(Hkv)])


def make_kv(B, Hkv, N, D, dtype: str, seed: int = DEFAULT_SEED, device="cpu", pin=(False, False)):
    """K, V [B,Hkv,N,D] in ``dtype``.  ``pin=(k, v)`` returns that tensor in pinned host memory
    (the values are the same bits whichever place they end up in)."""
    tdt = TORCH_DTYPES[dtype]
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    ch = torch.from_numpy(outlier_channels(Hkv, D, seed)).to(dev)
    outs = []
    for t, pinned in zip(range(2), pin):
        gen.manual_seed(seed * 2 + t + 1)
        if pinned:
            dst = torch.empty((B, Hkv, N, D), dtype=tdt, pin_memory=True)
        else:
            dst = torch.empty((B, Hkv, N, D), dtype=tdt, device=dev)
        for b in range(B):
            for h in range(Hkv):
                x = torch.randn((N, D), generator=gen, device=dev, dtype=torch.float32)
                x[:, ch[h]] *= OUTLIER_SCALE
                dst[b, h].copy_(x.to(tdt))
        outs.append(dst)
    return outs[0], outs[1]


@dataclass
class QueryChain:
    """Per-query-head AR(1) chains on the unit sphere (see module docstring)."""
    B: int
    Hq: int
    D: int = 128
    rho: float | np.ndarray = 0.95
    seed: int = DEFAULT_SEED
    exact: bool = False
    q_norm: float = 1.0
    _rng: np.random.Generator = field(init=False, repr=False)
    _q: np.ndarray | None = field(init=False, default=None, repr=False)

    def __post_init__(self):
        self._rng = np.random.Generator(np.random.Philox(key=[self.seed, 0x9E37]))
        self.rho = np.broadcast_to(np.asarray(self.rho, dtype=np.float64), (self.Hq,)).copy()

    def next(self) -> np.ndarray:
        """Next q_t as float64 [B,Hq,D] (before rounding to 16 bits)."""
        e = self._rng.standard_normal((self.B, self.Hq, self.D)) / np.sqrt(self.D)
        if self._q is None:
            x = e
        else:
            if self.exact:
                e = e - (e * self._q).sum(-1, keepdims=True) * self._q
                e = e / np.linalg.norm(e, axis=-1, keepdims=True)
            r = self.rho[None, :, None]
            x = r * self._q + np.sqrt(1.0 - r * r) * e
        self._q = x / np.linalg.norm(x, axis=-1, keepdims=True)
        return self._q * self.q_norm


def per_head_rho(Hkv: int, lo: float, hi: float, seed: int) -> np.ndarray:
    """One correlation per KV head, uniform over [lo, hi]: the Hkv equally spaced quantiles from lo to hi (both
    ends included), handed to the heads in a seeded random order.  Eight independent draws can miss a whole
    part of the range (with the default seed: everything above 0.84), and a threshold sweep over 0.8 - 0.95
    would then see no head that ever reuses; the quantiles cover the range whatever the seed."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 0x51D0]))
    grid = np.linspace(lo, hi, Hkv) if Hkv > 1 else np.array([0.5 * (lo + hi)])
    return grid[rng.permutation(Hkv)]


def chain_for(w: Workload, **kw) -> QueryChain:
    """The query chains of a workload.  With ``rho_range`` every KV head draws its own correlation and the
    query heads of its group share it (each still runs its own chain): the cache, its gate and its reuse
    rate are per KV head, so this is what makes reuse rates differ from head to head."""
    rho = np.repeat(per_head_rho(w.Hkv, *w.rho_range, w.seed), w.G) if w.rho_range else w.rho
    return QueryChain(w.B, w.Hq, w.D, rho, w.seed, **kw)


def round_to(x: np.ndarray, dtype: str) -> torch.Tensor:
    """float64 array -> torch tensor of the 16-bit dtype (round to nearest even, once)."""
    return torch.from_numpy(np.ascontiguousarray(x)).to(TORCH_DTYPES[dtype])


def bits(t: torch.Tensor) -> np.ndarray:
    """The uint16 bit patterns of a 16-bit float tensor, as a numpy array on the host."""
    assert t.dtype in (torch.float16, torch.bfloat16)
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def from_bits(a: np.ndarray, dtype: str) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(TORCH_DTYPES[dtype])
