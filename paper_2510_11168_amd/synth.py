"""Seeded synthetic inputs for the classifier-head step.

Holds input generation only -- none of the method's arithmetic (no rounding rule of the method,
no random-rounding stream, no gradients).  Both the tests' CPU oracle and the HIP path are fed
from here.  The shapes follow the public extreme-classification benchmarks the paper trains on
(its dataset-statistics table): embedding width 768, 1e5 .. 3e6 labels, a handful of positives
per sample drawn from a long-tailed (Zipf) label distribution.  The datasets themselves are not
used; these inputs stand in for them.
"""
from __future__ import annotations

import dataclasses

import numpy as np
import torch

BF16 = 0
E4M3 = 1
FLAG_SR = 1
FLAG_KAHAN = 2


@dataclasses.dataclass(frozen=True)
class HeadConfig:
    name: str
    cfg_id: int
    L: int
    d: int
    B: int
    chunk: int
    fmt: int
    flags: int
    zipf_s: float
    count_rule: str   # "fixed5" | "lognormal5" | "poisson4.5" | "poisson7"
    steps: int
    lr: float = 0.05
    w_std: float = 0.02


CONFIGS = {
    "tiny": HeadConfig("tiny", 1, 8192, 256, 64, 2048, BF16, FLAG_SR, 1.1, "fixed5", 3),
    "mid": HeadConfig("mid", 2, 131072, 768, 256, 32768, BF16, FLAG_KAHAN, 1.0, "lognormal5", 20),
    "large": HeadConfig("large", 3, 670091, 768, 512, 65536, BF16, FLAG_SR, 1.0, "poisson4.5", 50),
    "xl": HeadConfig("xl", 4, 3000000, 768, 1024, 131072, E4M3, FLAG_SR | FLAG_KAHAN, 1.05,
                     "poisson7", 20),
}


def xl_sweep(B: int, chunk: int, kahan: bool) -> HeadConfig:
    """The bandwidth-regime sweep points at 3M labels (E4M3 weights, SR)."""
    flags = FLAG_SR | (FLAG_KAHAN if kahan else 0)
    return HeadConfig(f"xl_B{B}_n{chunk}{'_kahan' if kahan else ''}", 5, 3000000, 768, B, chunk,
                      E4M3, flags, 1.05, "poisson7", 20)


def rng_for(cfg_id: int, step: int, data_seed: int = 0) -> np.random.Generator:
    return np.random.default_rng([data_seed, cfg_id, step])


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float array -> BF16 bit patterns via torch's CPU cast (a library cast, round to nearest)."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def make_x(rng: np.random.Generator, B: int, d: int) -> np.ndarray:
    """Encoder outputs: i.i.d. N(0,1) rows, L2-normalised in FP64, returned as BF16 bits [B, d]."""
    x = rng.standard_normal((B, d))
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    return to_bf16_bits(x)


def make_w0_f32(rng: np.random.Generator, n: int, d: int, std: float = 0.02) -> np.ndarray:
    """Initial weights N(0, std) as FP32 (the caller rounds them into the storage format)."""
    return (rng.standard_normal((n, d)) * std).astype(np.float32)


class ZipfLabels:
    """Rank-frequency Zipf over label ids: P(id = r - 1) proportional to r^-s, r = 1..L."""

    def __init__(self, L: int, s: float):
        w = np.arange(1, L + 1, dtype=np.float64) ** (-s)
        self.cdf = np.cumsum(w)
        self.cdf /= self.cdf[-1]
        self.L = L

    def draw_counts(self, rng: np.random.Generator, B: int, rule: str) -> np.ndarray:
        if rule == "fixed5":
            return np.full(B, 5, dtype=np.int64)
        if rule == "lognormal5":
            return np.clip(np.rint(5.0 * np.exp(0.6 * rng.standard_normal(B))), 1, 20).astype(np.int64)
        if rule.startswith("poisson"):
            return 1 + rng.poisson(float(rule[len("poisson"):]), B).astype(np.int64)
        raise ValueError(rule)

    def draw_csr(self, rng: np.random.Generator, B: int, rule: str):
        """CSR (indptr int32 [B+1], indices int32 [nnz]); per row ids distinct and ascending."""
        counts = np.minimum(self.draw_counts(rng, B, rule), self.L)
        indptr = np.zeros(B + 1, dtype=np.int32)
        rows = []
        for i in range(B):
            want = int(counts[i])
            got = np.zeros(0, dtype=np.int64)
            while len(got) < want:
                u = rng.random(2 * want)
                ids = np.minimum(np.searchsorted(self.cdf, u, side="left"), self.L - 1)
                got = np.unique(np.concatenate([got, ids]))
                if len(got) > want:
                    got = np.sort(rng.choice(got, size=want, replace=False))
            rows.append(got.astype(np.int32))
            indptr[i + 1] = indptr[i] + want
        return indptr, np.concatenate(rows).astype(np.int32)


def make_batch(cfg: HeadConfig, step: int, zipf: ZipfLabels | None = None, B: int | None = None):
    """One fresh batch (X bits, indptr, indices) for training step `step` of `cfg`."""
    rng = rng_for(cfg.cfg_id, step)
    B = cfg.B if B is None else B
    zipf = zipf or ZipfLabels(cfg.L, cfg.zipf_s)
    X = make_x(rng, B, cfg.d)
    indptr, indices = zipf.draw_csr(rng, B, cfg.count_rule)
    return X, indptr, indices
