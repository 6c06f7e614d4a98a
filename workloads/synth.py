"""Seeded synthetic activation matrices shaped like the paper's fine-tuning workloads.

The paper measures on LLaMA2-7B and ViT-B/16 activations (Section 4.1); those models and
datasets are not available, so every matrix here is a synthetic stand-in with the same shape
and a long-tailed singular spectrum as described in Section 2 (a dominant leading singular
value, a slowly decaying bulk, a small dense noise floor).

Everything is generated on the CPU with numpy's PCG64 from an integer seed, so the CPU oracle
and the GPU library see bit-identical inputs.  Matrices destined for the bf16 path are rounded
to bf16 (round-to-nearest-even) here and returned both as float32 values (exactly
representable in bf16) and as the raw uint16 bit patterns for upload.

No arithmetic of the decomposition itself lives in this module.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, Optional

import numpy as np

# ----------------------------------------------------------------------------- bf16 helpers


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to bf16 (nearest, ties to even); returns the uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounding = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + rounding) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen uint16 bf16 bit patterns to float32 (exact)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 array whose values are exactly representable in bf16."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x))


# ----------------------------------------------------------------------------- building blocks


def _orthonormal(rng: np.random.Generator, rows: int, cols: int) -> np.ndarray:
    """rows x cols matrix with orthonormal columns (thin QR of a Gaussian, signs fixed)."""
    g = rng.standard_normal((rows, cols))
    q, r = np.linalg.qr(g)
    q *= np.sign(np.diag(r))[None, :]
    return q


def spectrum_matrix(m: int, n: int, s: np.ndarray, noise: float, seed: int,
                    p_max: int = 1024) -> np.ndarray:
    """X = c * U diag(s) V^T + noise * N   (float64).

    U (m x p) and V (n x p) have orthonormal columns, p = min(m, n, len(s), p_max) leading
    terms of the spectrum are kept, c = sqrt(m n) / ||s||_2 gives the signal unit RMS so that
    `noise` is a relative noise level, and N is i.i.d. standard normal.
    """
    rng = np.random.default_rng(seed)
    p = int(min(m, n, len(s), p_max))
    s = np.asarray(s[:p], dtype=np.float64)
    c = np.sqrt(float(m) * float(n)) / np.linalg.norm(s)
    u = _orthonormal(rng, m, p)
    v = _orthonormal(rng, n, p)
    x = (u * (c * s)[None, :]) @ v.T
    if noise:
        x += noise * rng.standard_normal((m, n))
    return x


def spectrum_rank_k_floor(m: int, n: int, s: np.ndarray, noise: float, k: int,
                          p_max: int = 1024) -> float:
    """What the generator's own spectrum says a rank-k approximation of `spectrum_matrix(...)`
    can reach, relative to ||X||_F: cutting the signal after k terms leaves
    sqrt(c^2 sum_{i>k} s_i^2 + noise^2 m n), an upper bound on (and, the noise being far below
    the kept terms, an estimate of) the Eckart-Young optimum.  Expected values over the noise."""
    p = int(min(m, n, len(s), p_max))
    s = np.asarray(s[:p], dtype=np.float64)
    c2 = float(m) * float(n) / float(np.sum(s * s))
    noise2 = noise * noise * float(m) * float(n)
    return float(np.sqrt((c2 * np.sum(s[k:] ** 2) + noise2) / (c2 * np.sum(s * s) + noise2)))


def low_rank_plus_noise(m: int, n: int, rank: int, noise: float, seed: int) -> np.ndarray:
    """X = A B + noise * N with A (m x rank), B (rank x n), N all i.i.d. N(0,1) (float64)."""
    rng = np.random.default_rng(seed)
    a = rng.standard_normal((m, rank))
    b = rng.standard_normal((rank, n))
    x = a @ b
    if noise:
        x += noise * rng.standard_normal((m, n))
    return x


# ----------------------------------------------------------------------------- workloads


@dataclass
class Workload:
    """One activation site: the matrix the GPU sees, and the parameters of the call."""

    name: str
    x: np.ndarray                      # float32, values exactly representable in `dtype`
    dtype: str                         # "f32" or "bf16"
    k: int                             # target rank
    seed: int                          # seed handed to the decomposition (row sampling)
    extras: Dict[str, object] = field(default_factory=dict)

    @property
    def m(self) -> int:
        return int(self.x.shape[0])

    @property
    def n(self) -> int:
        return int(self.x.shape[1])

    @property
    def nbytes(self) -> int:
        return self.m * self.n * (2 if self.dtype == "bf16" else 4)

    def x_bits(self) -> np.ndarray:
        """Upload form: uint16 bf16 patterns, or the float32 array itself."""
        return f32_to_bf16_bits(self.x) if self.dtype == "bf16" else self.x


def _finish(name: str, x64: np.ndarray, dtype: str, k: int, seed: int, **extras) -> Workload:
    x32 = x64.astype(np.float32)
    if dtype == "bf16":
        x32 = round_to_bf16(x32)
    return Workload(name=name, x=x32, dtype=dtype, k=k, seed=seed, extras=dict(extras))


def c1_lowrank_f32(m: int = 1024, n: int = 256, rank: int = 16, seed: int = 0) -> Workload:
    """Config 1: fp32, exactly rank-`rank` signal plus 1e-3 Gaussian noise, k = rank."""
    return _finish("c1_lowrank_f32_%dx%d_k%d" % (m, n, rank),
                   low_rank_plus_noise(m, n, rank, 1e-3, seed), "f32", rank, seed)


def c2_vit(m: int = 64 * 197, n: int = 768, k: int = 32, seed: int = 2) -> Workload:
    """Config 2: ViT-B/16-shaped (64 images x 197 tokens), s_i = 0.9^i over 768 terms, bf16.

    The 3072-wide MLP-hidden site uses the same 768 spectrum values (zero beyond) with k = 64.
    """
    s = 0.9 ** np.arange(768)
    return _finish("c2_vit_%dx%d_k%d" % (m, n, k),
                   spectrum_matrix(m, n, s, 1e-3, seed), "bf16", k, seed,
                   rank_k_floor=spectrum_rank_k_floor(m, n, s, 1e-3, k))


def c3_llama(m: int = 4 * 2048, n: int = 4096, k: int = 128, seed: int = 3,
             n_out: Optional[int] = None, r_lora: int = 16) -> Workload:
    """Config 3: LLaMA-7B pre-norm activation (batch 4 x seq 2048), s_i = i^-1.5, bf16.

    Also carries the backward-side operands of the LoRA weight-gradient contraction: an
    upstream gradient dY (m x n_out, N(0,1), bf16), the LoRA up-projection B_lora
    (r_lora x n_out, N(0, 1/r_lora), bf16) and scale 1.
    """
    s = np.arange(1, n + 1, dtype=np.float64) ** -1.5
    n_out = n if n_out is None else n_out
    rng = np.random.default_rng(seed + 1000)
    dy = round_to_bf16(rng.standard_normal((m, n_out)).astype(np.float32))
    b = round_to_bf16((rng.standard_normal((r_lora, n_out)) / np.sqrt(r_lora)).astype(np.float32))
    return _finish("c3_llama_%dx%d_k%d" % (m, n, k),
                   spectrum_matrix(m, n, s, 1e-3, seed), "bf16", k, seed,
                   dY=dy, B_lora=b, r_lora=r_lora, scale=1.0,
                   rank_k_floor=spectrum_rank_k_floor(m, n, s, 1e-3, k))


def c4_mlp(m: int = 4 * 2048, n: int = 11008, k: int = 256, seed: int = 4,
           oversample: int = 8, power_iters: int = 1) -> Workload:
    """Config 4: LLaMA-7B MLP intermediate activation, s_i = exp(-i/64), bf16.

    Carries the RSVD comparator's parameters (oversampling 8, one power iteration).
    """
    s = np.exp(-np.arange(n, dtype=np.float64) / 64.0)
    return _finish("c4_mlp_%dx%d_k%d" % (m, n, k),
                   spectrum_matrix(m, n, s, 1e-3, seed), "bf16", k, seed,
                   oversample=oversample, power_iters=power_iters,
                   rank_k_floor=spectrum_rank_k_floor(m, n, s, 1e-3, k))


def c5_site_seed(layer: int, site: int) -> int:
    """Per-site seed of the long-context stream (32 layers x 7 sites)."""
    return 50_000 + 7 * int(layer) + int(site)


def c5_long_context_site(layer: int = 0, site: int = 0, m: int = 16 * 4096,
                         n: Optional[int] = None, k: int = 256) -> Workload:
    """Config 5: one site of the long-context stream (16 x 4096 tokens), s_i = i^-1.5, bf16.

    Sites 0..5 of a layer are 4096 wide (q/k/v/o inputs, gate/up input), site 6 is the
    11008-wide down-projection input.
    """
    if n is None:
        n = 11008 if site == 6 else 4096
    seed = c5_site_seed(layer, site)
    s = np.arange(1, n + 1, dtype=np.float64) ** -1.5
    return _finish("c5_L%d_S%d_%dx%d_k%d" % (layer, site, m, n, k),
                   spectrum_matrix(m, n, s, 1e-3, seed), "bf16", k, seed)


def coherent_activations(m: int = 8192, n: int = 4096, k: int = 128, seed: int = 6,
                         outlier_rows: int = 8, outlier_scale: float = 100.0,
                         dtype: str = "bf16") -> Workload:
    """Second workload: activations with outlier tokens (Section 2 reports a leading singular
    value above 1e4 against a bulk of 1e0..1e2; Theorem 4.3 ties the sampling error to the
    coherence of the leading singular vectors).

    The config-3 recipe plus `outlier_rows` seeded rows that each receive their own direction:
    row r_j += outlier_scale * sqrt(n) * w_j with w_j a random unit vector, i.e. `outlier_scale`
    times the RMS row norm of the bulk in a direction no other row shares.  The leading singular
    vectors then sit on single rows (coherence at its maximum m/k) and the leading singular values
    are ~outlier_scale times the bulk's.  Uniform row sampling sees such a row with probability
    k/m only and cannot recover its direction from the others, which is the regime where it is
    expected to lose against a Gaussian test matrix.  extras: the outlier row ids.
    """
    s = np.arange(1, min(m, n) + 1, dtype=np.float64) ** -1.5
    x = spectrum_matrix(m, n, s, 1e-3, seed)
    rng = np.random.default_rng(seed + 1000)
    rows = np.sort(rng.choice(m, size=outlier_rows, replace=False))
    w = rng.standard_normal((outlier_rows, n))
    w /= np.linalg.norm(w, axis=1, keepdims=True)
    x[rows, :] += outlier_scale * np.sqrt(n) * w
    return _finish("coherent_%dx%d_k%d" % (m, n, k), x, dtype, k, seed, outlier_rows=rows)


def exact_rank(m: int, n: int, rank: int, seed: int, dtype: str = "f32") -> Workload:
    """Exactly rank-`rank` matrix (no noise) with small-integer factors, so that the product
    is exact in fp32 and the matrix the GPU sees has exactly that rank."""
    rng = np.random.default_rng(seed)
    a = rng.integers(-3, 4, size=(m, rank)).astype(np.float64)
    b = rng.integers(-3, 4, size=(rank, n)).astype(np.float64)
    return _finish("exact_rank_%dx%d_r%d" % (m, n, rank), a @ b, dtype, rank, seed)


def gaussian_test_matrix(rows: int, cols: int, seed: int) -> np.ndarray:
    """i.i.d. N(0,1) matrix (float64) for callers that hand RSVD its test matrix as data."""
    return np.random.default_rng(seed).standard_normal((rows, cols))


FULL_SIZE: Dict[str, Callable[[], Workload]] = {
    "c1": c1_lowrank_f32,
    "c2a": lambda: c2_vit(n=768, k=32),
    "c2b": lambda: c2_vit(n=3072, k=64, seed=22),
    "c3": c3_llama,
    "c4": c4_mlp,
    "c5": c5_long_context_site,
    "coherent": coherent_activations,
}
