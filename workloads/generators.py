"""Synthetic low-rank hidden states, start blocks and projection weights.

Recipe (stand-in for the BERT / Llama-2 hidden states the paper measures on,
which need pretrained weights and public datasets that are not available
offline; only the layer shapes of Tab.2 and the low-rank structure shown in
Fig.1 / Fig.5 are taken from the paper):

    X_b = U_b · diag(s) · V_bᵀ + sigma · N_b

with U_b (L×n_s), V_b (d×n_s) the Q factors of seeded Gaussian matrices (for batch
items b > 0: the same factors with rows permuted and component signs flipped),
N_b ~ N(0,1) i.i.d. per entry, `sigma` a per-entry standard deviation, and `s`
one of the spectra below.  Start block Omega ~ N(0,1), d×r.  Weights
W ~ N(0, 1/d).  Everything is drawn with numpy's `default_rng(seed)` in
float64, then rounded once (round-to-nearest-even) to the storage type of the
call; the oracle consumes the rounded values upcast to float64, so input
quantisation never counts as error.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

BASE_SEED = 240302352


def config_seed(config: int, point: int = 0, b: int = 0) -> int:
    return BASE_SEED + 1000 * config + 10 * point + b


# --------------------------------------------------------------------------- #
# rounding helpers (storage only; no method arithmetic)
# --------------------------------------------------------------------------- #
def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float array to bfloat16 (RNE) and return it as float32 values."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(f.shape)


def round_to_dtype(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round to the storage dtype ("f32" or "bf16"); result is float32-valued."""
    if dtype == "bf16":
        return round_to_bf16(a)
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    raise ValueError(dtype)


# --------------------------------------------------------------------------- #
# spectra
# --------------------------------------------------------------------------- #
def _unit_rms(s: np.ndarray, L: int, d: int) -> np.ndarray:
    """Scale s so that U diag(s) Vᵀ has unit-RMS entries: sum s² = L·d."""
    return s * np.sqrt(L * d / np.sum(s * s))


def spectrum(kind: str, n: int, L: int, d: int, **kw) -> np.ndarray:
    """Singular values s_1 ≥ … ≥ s_n of the constructed signal.

    kinds: "geometric" (s_i = s0·q^i, i from 0), "exp" (unit-RMS,
    s_i ∝ exp(-i/tau), i from 0), "power" (unit-RMS, s_i ∝ i^-alpha, i from 1),
    "linear" (unit-RMS, falls linearly from c to c/2 over the n components),
    "flat" (all equal, unit-RMS).
    """
    if kind == "geometric":
        return kw.get("s0", 10.0) * kw.get("q", 0.8) ** np.arange(n, dtype=np.float64)
    if kind == "exp":
        return _unit_rms(np.exp(-np.arange(n, dtype=np.float64) / kw.get("tau", 48.0)), L, d)
    if kind == "power":
        return _unit_rms(np.arange(1, n + 1, dtype=np.float64) ** (-kw.get("alpha", 1.2)), L, d)
    if kind == "linear":
        t = np.arange(n, dtype=np.float64) / max(n - 1, 1)
        return _unit_rms(1.0 - 0.5 * t, L, d)
    if kind == "flat":
        return _unit_rms(np.ones(n, dtype=np.float64), L, d)
    raise ValueError(kind)


# --------------------------------------------------------------------------- #
# matrices
# --------------------------------------------------------------------------- #
def _orthonormal(rng: np.random.Generator, n: int, k: int) -> np.ndarray:
    q, _ = np.linalg.qr(rng.standard_normal((n, k)))
    return q


_FACTOR_CACHE: dict = {}


def _factors(L: int, d: int, n_s: int, seed: int):
    key = (L, d, n_s, seed)
    if key not in _FACTOR_CACHE:
        rng = np.random.default_rng(seed)
        _FACTOR_CACHE.clear()                       # keep one entry: the matrices are large
        _FACTOR_CACHE[key] = (_orthonormal(rng, L, n_s), _orthonormal(rng, d, n_s))
    return _FACTOR_CACHE[key]


def make_X(L: int, d: int, s: np.ndarray, sigma: float, seed: int,
           return_factors: bool = False, b: int = 0):
    """One hidden-state matrix X (L×d, float64) with singular spectrum ≈ s.

    The orthonormal factors (the costly part: two QR factorisations) are drawn once per
    `seed`; batch item b > 0 uses the same factors with their rows permuted and the
    components' signs flipped by a generator seeded with seed + b, which keeps them exactly
    orthonormal, and its own Gaussian noise."""
    n_s = len(s)
    U, V = _factors(L, d, n_s, seed)
    rng = np.random.default_rng(seed + 1_000_003 * (b + 1))
    if b > 0:
        U = U[rng.permutation(L)] * rng.choice([-1.0, 1.0], size=n_s)[None, :]
        V = V[rng.permutation(d)]
    X = (U * s) @ V.T
    if sigma > 0:
        X = X + sigma * rng.standard_normal((L, d))
    if return_factors:
        return X, U, V
    return X


def make_omega(d: int, r: int, seed: int) -> np.ndarray:
    """Start block Omega ~ N(0,1), d×r, float32 (shared by oracle and GPU)."""
    return np.random.default_rng(seed + 7).standard_normal((d, r)).astype(np.float32)


def make_weight(k: int, n: int, seed: int, fan_in: Optional[int] = None) -> np.ndarray:
    """Projection weight W ~ N(0, 1/fan_in), k×n, float64."""
    fan_in = k if fan_in is None else fan_in
    return np.random.default_rng(seed).standard_normal((k, n)) / np.sqrt(fan_in)


# --------------------------------------------------------------------------- #
# the five workloads
# --------------------------------------------------------------------------- #
@dataclass
class Workload:
    name: str
    config: int
    batch: int
    L: int
    d: int
    heads: int
    r: int
    dtype: str
    iters: int
    spec_kind: str
    spec_n: int
    spec_kw: dict = field(default_factory=dict)
    sigma: float = 0.0
    sigma_rel_s0: bool = False   # sigma given as a multiple of s_1
    ffn: int = 0                 # SwiGLU inner width (0 = no FFN on bases)
    out_proj: bool = True

    @property
    def d_head(self) -> int:
        return self.d // self.heads

    def s(self) -> np.ndarray:
        return spectrum(self.spec_kind, self.spec_n, self.L, self.d, **self.spec_kw)

    def noise(self) -> float:
        return self.sigma * (self.s()[0] if self.sigma_rel_s0 else 1.0)

    def X(self, b: int = 0, point: int = 0, return_factors: bool = False):
        return make_X(self.L, self.d, self.s(), self.noise(),
                      config_seed(self.config, point, 0), return_factors, b)

    def omega(self, point: int = 0) -> np.ndarray:
        return make_omega(self.d, self.r, config_seed(self.config, point, 0))

    def weight(self, which: str) -> np.ndarray:
        """which ∈ q,k,v,o,gate,up,down; float64, [in, out]."""
        base = BASE_SEED + 1000 * self.config + 500
        idx = ["q", "k", "v", "o", "gate", "up", "down"].index(which)
        d, f = self.d, self.ffn
        shp = {"q": (d, d), "k": (d, d), "v": (d, d), "o": (d, d),
               "gate": (d, f), "up": (d, f), "down": (f, d)}[which]
        return make_weight(shp[0], shp[1], base + idx)


CONFIGS = {
    # config 1: tiny fp32 case, single head
    "tiny": Workload("tiny", 1, 1, 128, 64, 1, 32, "f32", 4,
                     "geometric", 32, {"s0": 10.0, "q": 0.8}, 1e-3, out_proj=False),
    # config 2: BERT-base layer shape (Tab.2), r = L/2 and L/4
    "bert_r256": Workload("bert_r256", 2, 32, 512, 768, 12, 256, "bf16", 2,
                          "exp", 512, {"tau": 48.0}, 1e-2, sigma_rel_s0=True),
    "bert_r128": Workload("bert_r128", 2, 32, 512, 768, 12, 128, "bf16", 2,
                          "exp", 512, {"tau": 48.0}, 1e-2, sigma_rel_s0=True),
    # config 3: Llama-2-7B layer shape (Tab.2), r = L/4, FFN on bases
    "llama7b": Workload("llama7b", 3, 4, 4096, 4096, 32, 1024, "bf16", 2,
                        "power", 4096, {"alpha": 1.2}, 1e-3, ffn=11008),
    # config 4: long context, exact rank-1536 signal + tiny noise
    "long32k": Workload("long32k", 4, 1, 32768, 4096, 32, 2048, "bf16", 2,
                        "linear", 1536, {}, 1e-4),
}


def sweep_point(L: int, r_frac: int, alpha: float, sigma: float, iters: int) -> Workload:
    """Config 5 sweep point at the Llama-7B width (d=4096, 32 heads, batch 1)."""
    d = 4096
    return Workload(f"sweep_L{L}_r{r_frac}_a{alpha}_s{sigma}_k{iters}", 5, 1, L, d, 32,
                    L // r_frac, "bf16", iters, "power", min(L, d), {"alpha": alpha}, sigma)
