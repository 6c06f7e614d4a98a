"""fp64 CPU oracle for the LoRAct compression hot path.  TEST INFRASTRUCTURE ONLY.

This module is the slow, plain reference the GPU library is checked against.  It shares no
code with the HIP path and must never be imported by the product package: only the tests,
the smoke check and the benchmark's `cpu_baseline` leg call it.

What it follows (all citations are to the LoRAct paper, arXiv 2509.23472):

* `decompose`        Section 3.2, Algorithm 1 (sampling-based orthogonal decomposition): the
                     sketch of A by its own sampled rows, optionally sharpened by t power
                     rounds, an orthonormal basis U of the sketch's range, and V = U^T A.
* `decompose_adaptive`  the same with the rank chosen by the retained-energy count of Section 2
                     (sum of singular values), measured inside the sketch.
* `reconstruct`      Section 3.1, Eq. (4): A~ = U V.
* `lora_grad`        Section 3.1, Eq. (4)-(5) applied to a LoRA down-projection: the weight
                     gradient contraction A~^T (dY B^T) * scale, with A~ rebuilt first exactly
                     as the paper prescribes.
* `rsvd`             Section 3.2: the randomized SVD the paper compares with (the same
                     procedure with a Gaussian test matrix in place of the sampled rows), optional
                     oversampling with truncation to rank k by an SVD of the small factor.
* `prenorm_forward`, `prenorm_backward`
                     Section 3.3, Eqs. (6)-(10): RMS pre-norm unit that stores Norm(X) only.

The method is an approximation (a randomized range finder), so there is no closed-form
result to reach; the oracle takes the algorithm's steps literally in float64.  Library
primitives used as steps: numpy matmul, and numpy's SVD for the small l x n factor when l > k
(`rsvd`, and `decompose` with more sampled rows than the rank).
The thin QR is written out (Householder reflections) so that it can be pinned against LAPACK.

Parity status: the paper prints no worked numerical example of the decomposition, so the
numeric values of U, V are *parity unpinned by the paper*; the oracle is pinned instead by
what the paper's mathematics fixes (tests/test_oracle_pins.py): Q^T Q = I, exact recovery of
rank <= k inputs (proof of Theorem 4.2, first case), the deterministic bound of Theorem 4.2
evaluated with a brute-force SVD, the Eckart-Young lower bound, the projector identity
A~ = P_Y A, l = k = m reproducing A, LAPACK agreement of the QR, published splitmix64 output
values for the index generator, and the Halko-Martinsson-Tropp expectation bound quoted in
Section 3.2 for `rsvd`.

Readings of points the paper leaves open (each also listed in the design notes):
  - rows are sampled uniformly WITHOUT replacement (Theorem 4.2 needs a full-row-rank
    Omega_1; duplicates would break it);
  - the sample is drawn by splitmix64 + Floyd's algorithm and sorted ascending;
  - t = 0 on the hot path; for t >= 1 only Y is orthonormalised, as Algorithm 1 writes it;
  - QR sign convention diag(R) >= 0; a rank-deficient Y still yields an orthonormal Q;
  - more sampled rows than the rank (l > k, the setting of Theorem 4.3): Q spans the l-column
    sketch and B = Q^T A is truncated to rank k by its SVD, as in `rsvd`.
"""
from __future__ import annotations

from typing import Optional, Sequence, Tuple

import numpy as np

_MASK64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15


# ----------------------------------------------------------------------------- sampling


def _splitmix64_output(z: int) -> int:
    """Output function of splitmix64 applied to an already advanced state."""
    z &= _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


def splitmix64_stream(seed: int, count: int) -> list:
    """First `count` outputs of the splitmix64 generator started at state `seed`."""
    out = []
    state = seed & _MASK64
    for _ in range(count):
        state = (state + _GOLDEN) & _MASK64
        out.append(_splitmix64_output(state))
    return out


def sample_indices(m: int, l: int, seed: int) -> np.ndarray:
    """Algorithm 1, step 1: l distinct row ids drawn uniformly from [0, m), ascending.

    Floyd's subset sampling driven by splitmix64(seed): for i = m-l .. m-1 draw
    j = next() mod (i+1); keep j unless already chosen, in which case keep i.
    Every l-subset is equally likely (up to the negligible modulo bias of a 64-bit draw).
    """
    if not (0 <= l <= m):
        raise ValueError("need 0 <= l <= m")
    draws = splitmix64_stream(seed, l)
    chosen = set()
    for step, i in enumerate(range(m - l, m)):
        j = draws[step] % (i + 1)
        chosen.add(i if j in chosen else j)
    return np.array(sorted(chosen), dtype=np.int64)


# ----------------------------------------------------------------------------- thin QR


def householder_qr(y: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Thin QR of an m x k matrix (m >= k) by Householder reflections, float64.

    Returns Q (m x k, orthonormal columns) and R (k x k, upper triangular, diag >= 0).
    A rank-deficient Y still gives an orthonormal Q (the reflections are orthogonal
    regardless of the data); its columns beyond rank(Y) are then an arbitrary completion.
    """
    r = np.array(y, dtype=np.float64, copy=True)
    m, k = r.shape
    if m < k:
        raise ValueError("thin QR needs m >= k")
    vs = []
    for j in range(k):
        x = r[j:, j]
        normx = np.linalg.norm(x)
        v = x.copy()
        if normx == 0.0:
            vs.append(None)
            continue
        alpha = -normx if x[0] >= 0 else normx          # avoids cancellation in v[0]
        v[0] -= alpha
        v /= np.linalg.norm(v)
        r[j:, j:] -= 2.0 * np.outer(v, v @ r[j:, j:])
        vs.append(v)
    q = np.zeros((m, k))
    q[np.arange(k), np.arange(k)] = 1.0
    for j in range(k - 1, -1, -1):
        v = vs[j]
        if v is not None:
            q[j:, :] -= 2.0 * np.outer(v, v @ q[j:, :])
    rk = np.triu(r[:k, :])
    sign = np.where(np.diag(rk) < 0, -1.0, 1.0)
    return q * sign[None, :], rk * sign[:, None]


# ----------------------------------------------------------------------------- Algorithm 1


def decompose(a: np.ndarray, k: int, t: int = 0, seed: int = 0,
              idx: Optional[Sequence[int]] = None, l: Optional[int] = None
              ) -> Tuple[np.ndarray, np.ndarray]:
    """Algorithm 1: U (m x k, orthonormal columns), V (k x n) with A ~= U V.

    `idx` overrides the seed-derived sample (l row ids); otherwise
    idx = sample_indices(m, l, seed).

    `l` is the number of sampled rows.  Algorithm 1 takes l = k (the default).  Theorem 4.3
    states its bound for a sample A_l of l rows with the test matrix Omega = A_l^T; the paper
    does not say how rank-k factors are then returned, so for l > k this follows the reading
    used for the randomized SVD it compares with: Q spans the l-column sketch, and the l x n
    factor B = Q^T A is cut to its k leading singular triplets,
    U = Q Ub[:, :k], V = diag(s[:k]) Vb^T[:k, :].
    """
    a = np.asarray(a, dtype=np.float64)
    m, n = a.shape
    if l is None:
        l = k
    if not (1 <= k <= l <= min(m, n)):
        raise ValueError("need 1 <= k <= l <= min(m, n)")
    rows = sample_indices(m, l, seed) if idx is None else np.asarray(idx, dtype=np.int64)
    if rows.shape != (l,):
        raise ValueError("need exactly l sampled rows")
    # The test matrix is the transposed block of sampled rows, so the sketch is A A_l^T (m x l).
    a_l = a[rows, :]
    y = a @ a_l.T
    # Each power round replaces the sketch by A A^T Q with Q an orthonormal basis of the current
    # sketch; only the sketch is re-orthonormalised, A^T Q is used as it comes.
    for _ in range(t):
        q, _ = householder_qr(y)
        y = a @ (a.T @ q)
    # Orthonormal basis of range(Y); Q Q^T is the orthogonal projector that U V applies to A.
    q, _ = householder_qr(y)
    b = q.T @ a
    if l == k:
        return q, b
    ub, s, vbt = np.linalg.svd(b, full_matrices=False)
    return q @ ub[:, :k], s[:k, None] * vbt[:k, :]


def decompose_adaptive(a: np.ndarray, k_max: int, energy: float, t: int = 0, seed: int = 0,
                       idx: Optional[Sequence[int]] = None, l: Optional[int] = None):
    """Algorithm 1 with the rank chosen from the data (the paper's Conclusion leaves adaptive rank
    selection to future work; the rule is the one Section 2 uses to measure how low-rank
    activations are: the number of kept dimensions when `energy` of the energy, i.e. of the sum
    of the singular values, is retained).

    Reading: the energy is measured inside the sketch.  With Q an orthonormal basis of the
    l-column sketch and s_1 >= ... >= s_l the singular values of B = Q^T A (those of the projected
    matrix Q Q^T A), the rank is the smallest k with s_1 + ... + s_k >= energy * (s_1 + ... + s_l),
    capped at k_max; the factors are then cut to that k as in `decompose` with l > k.  When every
    row is sampled (l = min(m, n)) this is exactly the count Section 2 reports for A itself.

    Returns (U, V, k, fractions) with U m x k, V k x n and fractions[j] = (s_1 + ... + s_{j+1}) /
    (s_1 + ... + s_l).
    """
    a = np.asarray(a, dtype=np.float64)
    m, n = a.shape
    if l is None:
        l = k_max
    if not (1 <= k_max <= l <= min(m, n)) or not (0.0 < energy <= 1.0):
        raise ValueError("need 1 <= k_max <= l <= min(m, n) and 0 < energy <= 1")
    rows = sample_indices(m, l, seed) if idx is None else np.asarray(idx, dtype=np.int64)
    if rows.shape != (l,):
        raise ValueError("need exactly l sampled rows")
    y = a @ a[rows, :].T
    for _ in range(t):
        q, _ = householder_qr(y)
        y = a @ (a.T @ q)
    q, _ = householder_qr(y)
    b = q.T @ a
    ub, s, vbt = np.linalg.svd(b, full_matrices=False)
    fractions = np.cumsum(s) / np.sum(s)
    reached = np.nonzero(fractions >= energy)[0]
    k = int(reached[0]) + 1 if reached.size else l
    k = min(k, k_max)
    return q @ ub[:, :k], s[:k, None] * vbt[:k, :], k, fractions


def reconstruct(u: np.ndarray, v: np.ndarray) -> np.ndarray:
    """Section 3.1, Eq. (4): the activation rebuilt in the backward pass, A~ = U V."""
    return np.asarray(u, dtype=np.float64) @ np.asarray(v, dtype=np.float64)


def lora_grad(u: np.ndarray, v: np.ndarray, dy: np.ndarray, b_lora: np.ndarray,
              scale: float = 1.0) -> np.ndarray:
    """Weight gradient of a LoRA down-projection fed by the compressed activation.

    For Z = X W^T + scale * (X A_lora^T) B_lora^T with A_lora (r x n) and B_lora stored as
    r x n_out, dL/dA_lora^T = X^T (dY B_lora^T) * scale (n x r).  Following Section 3.1,
    Eqs. (4)-(5), the saved activation X is replaced by its reconstruction A~ = U V, which
    is formed first, exactly as the paper states the backward pass.
    """
    a_tilde = reconstruct(u, v)
    g = np.asarray(dy, dtype=np.float64) @ np.asarray(b_lora, dtype=np.float64).T
    return (a_tilde.T @ g) * float(scale)


# ----------------------------------------------------------------------------- RSVD comparator


def gaussian_stream(seed: int, count: int) -> np.ndarray:
    """`count` standard normal deviates from a counter-based generator (float64).

    Element e (0-based) takes h = the (e+1)-th splitmix64 output of `seed`, splits it into
    u1 = (high32 + 1) / 2^32 in (0, 1] and u2 = low32 / 2^32 in [0, 1), and returns the
    Box-Muller deviate sqrt(-2 ln u1) cos(2 pi u2).  Being a pure function of (seed, e) it
    can be evaluated independently, in any order, on any device.
    """
    e = np.arange(1, count + 1, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = np.uint64(seed & _MASK64) + e * np.uint64(_GOLDEN)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    hi = (z >> np.uint64(32)).astype(np.float64)
    lo = (z & np.uint64(0xFFFFFFFF)).astype(np.float64)
    u1 = (hi + 1.0) / 4294967296.0
    u2 = lo / 4294967296.0
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def gaussian_omega_t(l: int, n: int, seed: int) -> np.ndarray:
    """Gaussian test matrix stored transposed, l x n row-major (row j = test vector j)."""
    return gaussian_stream(seed, l * n).reshape(l, n)


def rsvd(a: np.ndarray, k: int, oversample: int = 0, power_iters: int = 0,
         omega_t: Optional[np.ndarray] = None, seed: int = 0
         ) -> Tuple[np.ndarray, np.ndarray]:
    """Randomized SVD as the paper's comparator (Section 3.2), rank-k factors U (m x k), V (k x n).

    Same steps as Algorithm 1 with the sampled block replaced by a Gaussian test matrix
    Omega (n x l, l = k + oversample; passed as Omega^T, l x n, or generated from `seed`).
    With l > k the l x n factor B = Q^T A is truncated to its k leading singular triplets:
    U = Q Ub[:, :k], V = diag(s[:k]) Vb^T[:k, :].
    """
    a = np.asarray(a, dtype=np.float64)
    m, n = a.shape
    l = k + oversample
    if not (1 <= k and l <= min(m, n)):
        raise ValueError("need 1 <= k and k + oversample <= min(m, n)")
    if omega_t is None:
        omega_t = gaussian_omega_t(l, n, seed)
    omega_t = np.asarray(omega_t, dtype=np.float64)
    if omega_t.shape != (l, n):
        raise ValueError("omega_t must be l x n")
    y = a @ omega_t.T
    for _ in range(power_iters):
        q, _ = householder_qr(y)
        y = a @ (a.T @ q)
    q, _ = householder_qr(y)
    b = q.T @ a
    if l == k:
        return q, b
    ub, s, vbt = np.linalg.svd(b, full_matrices=False)
    return q @ ub[:, :k], s[:k, None] * vbt[:k, :]


# ----------------------------------------------------------------------------- pre-norm unit


def prenorm_forward(x: np.ndarray, gamma: np.ndarray, eps: float = 0.0
                    ) -> Tuple[np.ndarray, np.ndarray]:
    """Section 3.3, Eq. (7): A = X / RMS(X) * gamma row-wise; returns (A, RMS vector)."""
    x = np.asarray(x, dtype=np.float64)
    rms = np.sqrt(np.mean(x * x, axis=1) + eps)
    return x / rms[:, None] * np.asarray(gamma, dtype=np.float64)[None, :], rms


def prenorm_backward(a: np.ndarray, rms: np.ndarray, gamma: np.ndarray,
                     grad_a: np.ndarray) -> np.ndarray:
    """Section 3.3, Eqs. (8)-(10): gradient w.r.t. X recovered from the stored A = Norm(X).

    Xbar = A / gamma;  dXbar = dA * gamma;
    dX = (dXbar - Xbar * mean_j(dXbar * Xbar)) / RMS      (mean over the hidden dimension).
    """
    gamma = np.asarray(gamma, dtype=np.float64)[None, :]
    xbar = np.asarray(a, dtype=np.float64) / gamma
    dxbar = np.asarray(grad_a, dtype=np.float64) * gamma
    inner = np.mean(dxbar * xbar, axis=1, keepdims=True)
    return (dxbar - xbar * inner) / np.asarray(rms, dtype=np.float64)[:, None]


# ----------------------------------------------------------------------------- metrics


def rel_fro(x: np.ndarray, ref: np.ndarray) -> float:
    """||x - ref||_F / ||ref||_F in float64."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm(x - ref) / np.linalg.norm(ref))


def orthogonality_defect(q: np.ndarray) -> float:
    """Spectral norm of Q^T Q - I in float64."""
    q = np.asarray(q, dtype=np.float64)
    return float(np.linalg.norm(q.T @ q - np.eye(q.shape[1]), 2))
