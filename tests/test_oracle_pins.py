"""Pins for the fp64 CPU oracle: it is checked against what the paper and the mathematics fix,
never against itself.  Citations are to the LoRAct paper (arXiv 2509.23472).

The paper prints no worked numerical example of Algorithm 1, so the values of U and V are
parity unpinned by the paper; these tests bind every step by invariants, closed forms,
special cases and brute force on tiny inputs, and the last group shows that plausible
mistakes planted in the oracle are caught by them.
"""
import os

import numpy as np
import pytest

from oracle import loract_oracle as orc
from workloads import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_vectors(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([int(tok) for tok in line.split()])
    return rows


def _tiny(m, n, seed, decay=0.7):
    """Full-rank tiny matrix with a decaying spectrum."""
    s = decay ** np.arange(min(m, n))
    return synth.spectrum_matrix(m, n, s, 0.0, seed)


# ----------------------------------------------------------------------------- index generator


def test_splitmix64_matches_published_vectors():
    for row in _read_vectors("splitmix64_vectors.txt"):
        seed, expected = row[0], row[1:]
        assert orc.splitmix64_stream(seed, len(expected)) == expected


def test_sample_indices_hand_derived_vectors():
    for row in _read_vectors("sample_indices_vectors.txt"):
        m, l, seed, expected = row[0], row[1], row[2], row[3:]
        assert orc.sample_indices(m, l, seed).tolist() == expected


@pytest.mark.parametrize("m,l", [(1, 1), (5, 5), (17, 4), (1000, 37), (8192, 128)])
def test_sample_indices_distinct_sorted_in_range(m, l):
    for seed in range(5):
        idx = orc.sample_indices(m, l, seed)
        assert idx.shape == (l,)
        assert np.all(np.diff(idx) > 0)            # sorted and distinct: no replacement
        assert idx[0] >= 0 and idx[-1] < m


def test_sample_indices_uniform_chi_square():
    # Row sampling of Algorithm 1 / Theorem 4.3: *uniform* row sampling.  Every row of m = 20 should be
    # picked with probability l/m = 0.25; chi-square over 4000 seeds, 19 dof, 99.9% quantile 43.8.
    m, l, trials = 20, 5, 4000
    counts = np.zeros(m)
    for seed in range(trials):
        counts[orc.sample_indices(m, l, seed)] += 1
    expected = trials * l / m
    # variance of each count is that of a Bernoulli(l/m) sum, so scale accordingly
    chi2 = np.sum((counts - expected) ** 2 / (expected * (1 - l / m))) * (m - 1) / m
    assert chi2 < 43.8


# ----------------------------------------------------------------------------- thin QR


@pytest.mark.parametrize("m,k", [(8, 8), (40, 7), (300, 33)])
def test_householder_qr_invariants_and_lapack(m, k):
    rng = np.random.default_rng(m * 100 + k)
    y = rng.standard_normal((m, k)) * (10.0 ** rng.uniform(-3, 3, size=k))[None, :]
    q, r = orc.householder_qr(y)
    assert q.shape == (m, k) and r.shape == (k, k)
    assert np.linalg.norm(q.T @ q - np.eye(k), 2) <= 1e-12          # Algorithm 1: Q orthonormal
    assert np.linalg.norm(q @ r - y) <= 1e-12 * np.linalg.norm(y)    # Y = Q R
    assert np.allclose(r, np.triu(r)) and np.all(np.diag(r) >= 0)
    # thin QR with diag(R) > 0 is unique for full-column-rank Y: must agree with LAPACK
    ql, rl = np.linalg.qr(y)
    sg = np.sign(np.diag(rl))
    assert np.allclose(q, ql * sg[None, :], atol=1e-10)
    assert np.allclose(r, rl * sg[:, None], rtol=1e-10, atol=1e-10 * np.abs(rl).max())


def test_householder_qr_rank_deficient_still_orthonormal():
    rng = np.random.default_rng(5)
    y = rng.standard_normal((50, 3)) @ rng.standard_normal((3, 8))     # rank 3, 8 columns
    y[:, 5] = 0.0
    q, r = orc.householder_qr(y)
    assert np.linalg.norm(q.T @ q - np.eye(8), 2) <= 1e-12
    assert np.linalg.norm(q @ r - y) <= 1e-12 * np.linalg.norm(y)


# ----------------------------------------------------------------------------- Algorithm 1


@pytest.mark.parametrize("m,n,k,t", [(64, 24, 4, 0), (64, 24, 12, 0), (30, 50, 9, 0),
                                      (64, 24, 6, 1), (64, 24, 6, 2)])
def test_decompose_shapes_orthonormal_and_projection(m, n, k, t):
    a = _tiny(m, n, seed=m + n + k)
    for seed in range(4):
        u, v = orc.decompose(a, k, t=t, seed=seed)
        assert u.shape == (m, k) and v.shape == (k, n)               # Section 3.1: U m x k, V k x n
        assert orc.orthogonality_defect(u) <= 1e-12
        assert np.allclose(v, u.T @ a, atol=1e-12 * np.abs(a).max() * m)  # V = Q^T A


@pytest.mark.parametrize("m,n,k", [(64, 24, 4), (64, 24, 12), (30, 50, 9)])
def test_decompose_equals_orthogonal_projector_onto_range_of_sketch(m, n, k):
    # Theorem 4.2 speaks of P_Y A with P_Y the orthogonal projector onto range(Y), Y = A Omega,
    # Omega = A_k^T (Theorem 4.3).  Build P_Y from the pseudo-inverse, a route that shares
    # nothing with Householder QR.
    a = _tiny(m, n, seed=7 * m + k, decay=0.8)
    for seed in range(4):
        idx = orc.sample_indices(m, k, seed)
        omega = a[idx, :].T
        y = a @ omega
        p_y = y @ np.linalg.pinv(y)
        u, v = orc.decompose(a, k, seed=seed)
        assert np.allclose(orc.reconstruct(u, v), p_y @ a, atol=1e-9 * np.linalg.norm(a))


@pytest.mark.parametrize("rank,k", [(3, 3), (3, 5), (8, 8)])
def test_exact_recovery_when_rank_at_most_k(rank, k):
    # Proof of Theorem 4.2, first case: rank(A) <= k and Omega_1 of full row rank => error 0.
    rng = np.random.default_rng(rank * 10 + k)
    a = rng.standard_normal((60, rank)) @ rng.standard_normal((rank, 40))
    for seed in range(5):
        u, v = orc.decompose(a, k, seed=seed)
        assert orc.rel_fro(orc.reconstruct(u, v), a) <= 1e-12
        assert orc.orthogonality_defect(u) <= 1e-12


def test_sampling_every_row_reproduces_the_matrix():
    # l = k = m with A of full row rank: range(Y) = range(A A^T) = R^m, so P_Y A = A.
    a = _tiny(12, 30, seed=3, decay=0.9)
    u, v = orc.decompose(a, 12, seed=0)
    assert orc.rel_fro(orc.reconstruct(u, v), a) <= 1e-11


@pytest.mark.parametrize("m,n,k", [(64, 24, 4), (64, 24, 8), (64, 24, 12), (40, 60, 10)])
def test_theorem_4_2_bound_and_eckart_young(m, n, k):
    # Theorem 4.2 with Omega = A_k^T, every quantity from a brute-force SVD:
    #   ||A - P_Y A||_2^2 <= ||Sigma_2||^2 + ||Sigma_2 Omega_2 Omega_1^+||^2
    # and Eckart-Young (Section 3.2): no rank-k approximation beats the truncated SVD.
    a = _tiny(m, n, seed=11 * m + k, decay=0.75)
    _, s, vt = np.linalg.svd(a, full_matrices=False)
    v1, v2, s2 = vt[:k, :].T, vt[k:, :].T, s[k:]
    for seed in range(25):
        idx = orc.sample_indices(m, k, seed)
        omega = a[idx, :].T
        omega1, omega2 = v1.T @ omega, v2.T @ omega
        assert np.linalg.matrix_rank(omega1) == k
        bound = s2[0] ** 2 + np.linalg.norm((s2[:, None] * omega2) @ np.linalg.pinv(omega1), 2) ** 2
        u, v = orc.decompose(a, k, seed=seed)
        resid = a - orc.reconstruct(u, v)
        err2 = np.linalg.norm(resid, 2)
        assert err2 ** 2 <= bound * (1 + 1e-9)
        assert err2 >= s2[0] * (1 - 1e-9)
        assert np.linalg.norm(resid) >= np.sqrt(np.sum(s2 ** 2)) * (1 - 1e-9)


def test_closed_form_on_scaled_orthonormal_rows():
    # A = D W with W having orthonormal rows and D diagonal: A A_k^T = D W W_S^T D_S has
    # range span{e_i : i in S}, so P_Y A keeps exactly the sampled rows and zeroes the others.
    rng = np.random.default_rng(9)
    w = synth._orthonormal(rng, 40, 16).T              # 16 x 40, orthonormal rows
    d = np.arange(1, 17, dtype=np.float64)
    a = d[:, None] * w
    idx = orc.sample_indices(16, 5, seed=4)
    u, v = orc.decompose(a, 5, seed=4)
    expected = np.zeros_like(a)
    expected[idx, :] = a[idx, :]
    assert np.allclose(orc.reconstruct(u, v), expected, atol=1e-11)


def test_power_iterations_approach_truncated_svd():
    # Power rounds of Algorithm 1: with a spectral gap the range of (A A^T)^t A Omega converges to
    # the leading left singular subspace, so the error tends to the Eckart-Young optimum.
    rng = np.random.default_rng(21)
    s = np.concatenate([np.linspace(10, 5, 6), np.linspace(0.5, 0.1, 18)])
    a = (synth._orthonormal(rng, 80, 24) * s[None, :]) @ synth._orthonormal(rng, 30, 24).T
    best = np.sqrt(np.sum(s[6:] ** 2))
    errs = []
    for t in (0, 1, 2, 4):
        u, v = orc.decompose(a, 6, t=t, seed=1)
        errs.append(np.linalg.norm(a - orc.reconstruct(u, v)))
    assert errs[1] <= errs[0] and errs[3] <= errs[1]
    assert errs[3] <= best * (1 + 1e-3)
    assert all(e >= best * (1 - 1e-12) for e in errs)


def test_explicit_indices_override_seed():
    a = _tiny(40, 20, seed=2)
    idx = orc.sample_indices(40, 6, 123)
    u1, v1 = orc.decompose(a, 6, seed=123)
    u2, v2 = orc.decompose(a, 6, seed=999, idx=idx)
    assert np.array_equal(u1, u2) and np.array_equal(v1, v2)


# ----------------------------------------------------------------------------- consumers of the factors


def test_lora_grad_matches_finite_difference_of_loss():
    # The contraction is the gradient, w.r.t. the LoRA down-projection A_lora (r x n), of
    # L = sum(dY * Z), Z = scale * (X~ A_lora^T) B_lora^T, with X~ = U V (Section 3.1 Eq. 4-5).
    rng = np.random.default_rng(4)
    m, n, n_out, r, k, scale = 30, 12, 10, 3, 5, 0.7
    a = _tiny(m, n, seed=8)
    u, v = orc.decompose(a, k, seed=0)
    dy = rng.standard_normal((m, n_out))
    b = rng.standard_normal((r, n_out))
    a_lora = rng.standard_normal((r, n))
    x_t = orc.reconstruct(u, v)

    def loss(al):
        return float(np.sum(dy * (scale * (x_t @ al.T) @ b)))

    g = orc.lora_grad(u, v, dy, b, scale)              # n x r
    assert g.shape == (n, r)
    h = 1e-6
    for (i, j) in [(0, 0), (5, 2), (11, 1)]:
        e = np.zeros_like(a_lora)
        e[j, i] = h
        fd = (loss(a_lora + e) - loss(a_lora - e)) / (2 * h)
        assert abs(fd - g[i, j]) <= 1e-6 * max(1.0, abs(fd))


def test_prenorm_backward_matches_finite_difference():
    # Section 3.3, Eqs. (6)-(10): gradient through Norm recovered from A = Norm(X) and RMS only.
    rng = np.random.default_rng(12)
    m, n = 5, 9
    x = rng.standard_normal((m, n)) * 3.0
    gamma = rng.uniform(0.5, 2.0, size=n)
    grad_a = rng.standard_normal((m, n))
    a, rms = orc.prenorm_forward(x, gamma)
    assert np.allclose(rms, np.sqrt(np.mean(x ** 2, axis=1)))
    dx = orc.prenorm_backward(a, rms, gamma, grad_a)
    h = 1e-6
    for (i, j) in [(0, 0), (2, 5), (4, 8)]:
        e = np.zeros_like(x)
        e[i, j] = h
        fp = np.sum(grad_a * orc.prenorm_forward(x + e, gamma)[0])
        fm = np.sum(grad_a * orc.prenorm_forward(x - e, gamma)[0])
        assert abs((fp - fm) / (2 * h) - dx[i, j]) <= 1e-7


def test_prenorm_forward_closed_forms():
    # Eq. (7) pinned by what it must produce, not by retyping it:
    # (a) gamma = 1, eps = 0: every row of A has unit root-mean-square;
    rng = np.random.default_rng(12)
    m, n = 7, 24
    x = rng.standard_normal((m, n)) * rng.uniform(0.1, 30.0, size=(m, 1))
    a, rms = orc.prenorm_forward(x, np.ones(n))
    assert np.allclose(np.sum(a * a, axis=1), n, rtol=1e-13)
    # (b) the RMS vector times A / gamma gives X back (what the backward pass relies on, Eq. 8);
    gamma = rng.uniform(0.5, 2.0, size=n)
    a, rms = orc.prenorm_forward(x, gamma)
    assert np.allclose(a / gamma[None, :] * rms[:, None], x, rtol=1e-13)
    # (c) a row of +-c has RMS c and normalises to +-gamma; scaling a row leaves A unchanged;
    signs = np.where(rng.random(n) < 0.5, -1.0, 1.0)
    a1, r1 = orc.prenorm_forward(3.5 * signs[None, :], gamma)
    assert r1[0] == pytest.approx(3.5, rel=1e-15) and np.allclose(a1[0], signs * gamma, rtol=1e-15)
    a2, r2 = orc.prenorm_forward(17.0 * x, gamma)
    assert np.allclose(a2, a, rtol=1e-13) and np.allclose(r2, 17.0 * rms, rtol=1e-13)
    # (d) a worked row: x = (3, 4, 0, 0): mean square 25/4, RMS 5/2, A = (6/5, 8/5, 0, 0) gamma
    a3, r3 = orc.prenorm_forward(np.array([[3.0, 4.0, 0.0, 0.0]]), np.array([1.0, 2.0, 1.0, 1.0]))
    assert r3[0] == 2.5 and np.allclose(a3[0], [1.2, 3.2, 0.0, 0.0], rtol=1e-15)
    # (e) eps enters under the root: an all-zero row stays finite and maps to zero
    a4, r4 = orc.prenorm_forward(np.zeros((1, 4)), np.ones(4), eps=1e-6)
    assert r4[0] == pytest.approx(1e-3) and np.all(a4 == 0.0)


# ----------------------------------------------------------------------------- RSVD comparator


def test_gaussian_stream_moments_and_counter_property():
    g = orc.gaussian_stream(3, 200_000)
    assert abs(g.mean()) < 0.01 and abs(g.std() - 1) < 0.01
    assert abs(np.mean(g ** 3)) < 0.03 and abs(np.mean(g ** 4) - 3) < 0.1
    # element e is a pure function of (seed, e), built on the published splitmix64 outputs
    first = orc.splitmix64_stream(3, 1)[0]
    u1 = ((first >> 32) + 1) / 2.0 ** 32
    u2 = (first & 0xFFFFFFFF) / 2.0 ** 32
    assert g[0] == pytest.approx(np.sqrt(-2 * np.log(u1)) * np.cos(2 * np.pi * u2), rel=1e-14)
    assert np.array_equal(orc.gaussian_stream(3, 1000), g[:1000])
    assert np.array_equal(orc.gaussian_omega_t(4, 250, 3).ravel(), g[:1000])


def test_rsvd_exact_recovery_and_truncation():
    rng = np.random.default_rng(30)
    a = rng.standard_normal((50, 4)) @ rng.standard_normal((4, 35))
    for p in (0, 3):
        u, v = orc.rsvd(a, 4, oversample=p, seed=5)
        assert u.shape == (50, 4) and v.shape == (4, 35)
        assert orc.rel_fro(orc.reconstruct(u, v), a) <= 1e-11
        assert orc.orthogonality_defect(u) <= 1e-11
    # singular values of the truncated factor never exceed the true ones (interlacing)
    a = _tiny(60, 30, seed=6, decay=0.8)
    s_true = np.linalg.svd(a, compute_uv=False)
    u, v = orc.rsvd(a, 6, oversample=4, seed=1)
    s_apx = np.linalg.svd(v, compute_uv=False)
    assert np.all(s_apx <= s_true[:6] * (1 + 1e-12))


def test_rsvd_mean_error_within_quoted_bound():
    # Section 3.2 quotes E||A - Q Q^T A|| <= (1 + sqrt(k/(l-k))) s_{k+1} + e sqrt(l)/(l-k) sqrt(sum_{j>k} s_j^2)
    # for the Gaussian range finder with l columns.
    a = _tiny(80, 40, seed=14, decay=0.85)
    s = np.linalg.svd(a, compute_uv=False)
    k, p = 6, 4
    l = k + p
    bound = (1 + np.sqrt(k / (l - k))) * s[k] + np.e * np.sqrt(l) / (l - k) * np.sqrt(np.sum(s[k:] ** 2))
    errs = []
    for seed in range(60):
        q, b = orc.rsvd(a, l, oversample=0, seed=seed)       # the l-column range finder itself
        errs.append(np.linalg.norm(a - q @ b, 2))
    assert np.mean(errs) <= bound
    assert np.min(errs) >= s[l] * (1 - 1e-12)


def test_sampling_and_gaussian_sketches_are_comparable():
    # Section 3.2's qualitative claim: replacing the Gaussian test matrix by sampled rows keeps
    # the approximation quality comparable (no number is printed; O(1) ratio on an incoherent input).
    a = _tiny(120, 60, seed=77, decay=0.85)
    e_s = np.mean([np.linalg.norm(a - orc.reconstruct(*orc.decompose(a, 10, seed=s))) for s in range(30)])
    e_g = np.mean([np.linalg.norm(a - orc.reconstruct(*orc.rsvd(a, 10, seed=s))) for s in range(30)])
    assert 0.5 <= e_s / e_g <= 2.0


# ----------------------------------------------------------------------------- more sampled rows than the rank


@pytest.mark.parametrize("m,n,k,l", [(60, 28, 5, 9), (48, 40, 8, 16), (70, 30, 6, 7)])
def test_oversampled_decompose_is_best_rank_k_of_the_projected_matrix(m, n, k, l):
    # Theorem 4.3's setting (l >= k sampled rows, Omega = A_l^T).  With P the orthogonal projector
    # onto range(A A_l^T), built here from a least-squares solve and not from the oracle's QR,
    # the rank-k factors must multiply to the best rank-k approximation of P A (Eckart-Young,
    # Section 3.2), and the error splits by Pythagoras into the range-finder error plus the
    # discarded singular values of P A.
    a = _tiny(m, n, seed=3 * m + l, decay=0.8)
    for seed in range(4):
        idx = orc.sample_indices(m, l, seed)
        y = a @ a[idx, :].T
        pa = y @ np.linalg.lstsq(y, a, rcond=None)[0]
        ub, sb, vbt = np.linalg.svd(pa, full_matrices=False)
        best = (ub[:, :k] * sb[:k]) @ vbt[:k, :]
        u, v = orc.decompose(a, k, seed=seed, l=l)
        assert u.shape == (m, k) and v.shape == (k, n)
        assert orc.orthogonality_defect(u) <= 1e-11
        assert orc.rel_fro(u @ v, best) <= 1e-9
        lhs = np.linalg.norm(a - u @ v) ** 2
        rhs = np.linalg.norm(a - pa) ** 2 + np.sum(sb[k:l] ** 2)
        assert abs(lhs - rhs) <= 1e-9 * np.linalg.norm(a) ** 2


def test_oversampled_decompose_bounds_and_special_cases():
    rng = np.random.default_rng(41)
    # rank <= k input is recovered exactly whatever l (proof of Theorem 4.2, first case)
    a = rng.standard_normal((50, 4)) @ rng.standard_normal((4, 35))
    u, v = orc.decompose(a, 4, seed=2, l=9)
    assert orc.rel_fro(u @ v, a) <= 1e-11
    # l = k is Algorithm 1 itself
    a = _tiny(64, 24, seed=8, decay=0.75)
    u0, v0 = orc.decompose(a, 6, seed=3)
    u1, v1 = orc.decompose(a, 6, seed=3, l=6)
    assert np.array_equal(u0, u1) and np.array_equal(v0, v1)
    # deterministic bound of Theorem 4.2 with a k x l block Omega_1 (full row rank), plus at most
    # sigma_{k+1} for the truncation; and the Eckart-Young floor
    _, s, vt = np.linalg.svd(a, full_matrices=False)
    k, l = 6, 11
    v1t, v2t, s2 = vt[:k, :], vt[k:, :], s[k:]
    for seed in range(10):
        idx = orc.sample_indices(64, l, seed)
        omega = a[idx, :].T
        range_bound = np.sqrt(s2[0] ** 2 + np.linalg.norm((s2[:, None] * (v2t @ omega)) @ np.linalg.pinv(v1t @ omega), 2) ** 2)
        u, v = orc.decompose(a, k, seed=seed, l=l)
        err = np.linalg.norm(a - u @ v, 2)
        assert s[k] * (1 - 1e-12) <= err <= (s[k] + range_bound) * (1 + 1e-9)
        assert np.all(np.linalg.svd(v, compute_uv=False) <= s[:k] * (1 + 1e-12))
    # more sampled rows help on average
    e_k = np.mean([np.linalg.norm(a - np.matmul(*orc.decompose(a, k, seed=sd))) for sd in range(30)])
    e_2k = np.mean([np.linalg.norm(a - np.matmul(*orc.decompose(a, k, seed=sd, l=2 * k))) for sd in range(30)])
    assert e_2k < e_k


# ----------------------------------------------------------------------------- planted mistakes are caught


def _theorem_4_2_holds(decompose_fn, trials=10):
    m, n, k = 64, 24, 8
    a = _tiny(m, n, seed=11 * m + k, decay=0.75)
    _, s, vt = np.linalg.svd(a, full_matrices=False)
    v1, v2, s2 = vt[:k, :].T, vt[k:, :].T, s[k:]
    for seed in range(trials):
        idx = orc.sample_indices(m, k, seed)
        omega = a[idx, :].T
        bound = s2[0] ** 2 + np.linalg.norm((s2[:, None] * (v2.T @ omega)) @ np.linalg.pinv(v1.T @ omega), 2) ** 2
        u, v = decompose_fn(a, k, seed)
        if np.linalg.norm(a - u @ v, 2) ** 2 > bound * (1 + 1e-9):
            return False
    return True


def test_planted_mistakes_violate_the_pins():
    def correct(a, k, seed):
        return orc.decompose(a, k, seed=seed)

    def no_final_qr(a, k, seed):              # drops the final QR: U = normalised Y instead of Q
        idx = orc.sample_indices(a.shape[0], k, seed)
        y = a @ a[idx, :].T
        u = y / np.linalg.norm(y, axis=0, keepdims=True)
        return u, u.T @ a

    def sketch_without_transpose(a, k, seed):  # Y = A_k-based sketch from the wrong side
        idx = orc.sample_indices(a.shape[0], k, seed)
        y = np.zeros((a.shape[0], k))
        y[idx, np.arange(k)] = 1.0             # range = sampled coordinate axes, not range(A A_k^T)
        q, _ = orc.householder_qr(y)
        return q, q.T @ a

    def wrong_projection_sign(a, k, seed):
        u, v = orc.decompose(a, k, seed=seed)
        return u, -v

    assert _theorem_4_2_holds(correct)
    assert not _theorem_4_2_holds(no_final_qr)
    assert not _theorem_4_2_holds(sketch_without_transpose)
    assert not _theorem_4_2_holds(wrong_projection_sign)


def test_planted_truncation_mistakes_violate_the_oversampled_pin():
    # the check of test_oversampled_decompose_is_best_rank_k_of_the_projected_matrix, applied to
    # two plausible wrong truncations of the l-column basis
    m, n, k, l = 60, 28, 5, 9
    a = _tiny(m, n, seed=3 * m + l, decay=0.8)
    idx = orc.sample_indices(m, l, 0)
    y = a @ a[idx, :].T
    pa = y @ np.linalg.lstsq(y, a, rcond=None)[0]
    ub, sb, vbt = np.linalg.svd(pa, full_matrices=False)
    best = (ub[:, :k] * sb[:k]) @ vbt[:k, :]

    q, _ = orc.householder_qr(y)
    first_columns = q[:, :k] @ (q[:, :k].T @ a)            # keeps k columns of Q instead of k triplets of B
    b = q.T @ a
    ubb, sbb, vbbt = np.linalg.svd(b, full_matrices=False)
    unscaled = (q @ ubb[:, :k]) @ vbbt[:k, :]              # forgets the singular values in V
    good = np.matmul(*orc.decompose(a, k, seed=0, l=l))
    assert orc.rel_fro(good, best) <= 1e-9
    assert orc.rel_fro(first_columns, best) > 1e-3
    assert orc.rel_fro(unscaled, best) > 1e-3


# ----------------------------------------------------------------------------- adaptive rank


def _orthonormal_factors(m, n, r, seed):
    rng = np.random.default_rng(seed)
    u, _ = np.linalg.qr(rng.standard_normal((m, r)))
    v, _ = np.linalg.qr(rng.standard_normal((n, r)))
    return u, v


def test_adaptive_rank_worked_example():
    # A with singular values (3, 2, 1, 1, 1) exactly and l >= 5 sampled rows: the sketch spans the
    # whole row space, B = Q^T A has the singular values of A, and the retained fractions of the
    # energy (sum of singular values, Section 2) are 3/8, 5/8, 6/8, 7/8, 8/8.
    u, v = _orthonormal_factors(40, 30, 5, 1)
    a = (u * np.array([3.0, 2.0, 1.0, 1.0, 1.0])[None, :]) @ v.T
    for energy, want in [(0.3, 1), (0.375 - 1e-9, 1), (0.5, 2), (0.7, 3), (0.8, 4), (0.9, 5), (1.0 - 1e-9, 5)]:
        uu, vv, k, frac = orc.decompose_adaptive(a, 8, energy, seed=3, l=8)
        assert k == want, (energy, k)
        assert uu.shape == (40, k) and vv.shape == (k, 30)
        assert np.allclose(frac[:5], [3 / 8, 5 / 8, 6 / 8, 7 / 8, 1.0], atol=1e-12)
        # the factors are the k leading singular triplets of A itself here
        best = (u[:, :k] * np.array([3.0, 2.0, 1.0, 1.0, 1.0])[None, :k]) @ v[:, :k].T
        if want in (1, 2, 5):      # (the triple singular value 1 has no unique truncation in between)
            assert np.allclose(uu @ vv, best, atol=1e-10)
    # the cap: never more than k_max columns
    assert orc.decompose_adaptive(a, 3, 0.99, seed=3, l=8)[2] == 3


@pytest.mark.parametrize("m,n,l", [(60, 24, 10), (35, 50, 20)])
def test_adaptive_rank_is_the_count_on_the_projected_matrix(m, n, l):
    # brute force: singular values of P_Y A with P_Y from the pseudo-inverse of the sketch, no QR
    a = _tiny(m, n, 7)
    for seed in range(4):
        rows = orc.sample_indices(m, l, seed)
        y = a @ a[rows, :].T
        p_y = y @ np.linalg.pinv(y)
        s = np.linalg.svd(p_y @ a, compute_uv=False)[:l]
        for energy in (0.5, 0.8, 0.9, 0.97):
            want = int(np.nonzero(np.cumsum(s) / np.sum(s) >= energy)[0][0]) + 1
            uu, vv, k, _ = orc.decompose_adaptive(a, l, energy, seed=seed)
            assert k == want
            # and the factors are those of the fixed-rank call with that k
            u2, v2 = orc.decompose(a, k, seed=seed, l=l)
            assert np.allclose(uu @ vv, u2 @ v2, atol=1e-10 * np.abs(a).max())


def test_adaptive_rank_with_every_row_sampled_is_the_count_of_section_2():
    a = _tiny(18, 30, 5, decay=0.6)
    s = np.linalg.svd(a, compute_uv=False)
    ks = []
    for energy in (0.5, 0.9, 0.99):
        want = int(np.nonzero(np.cumsum(s) / np.sum(s) >= energy)[0][0]) + 1
        k = orc.decompose_adaptive(a, 18, energy, idx=np.arange(18))[2]
        assert k == want
        ks.append(k)
    assert ks == sorted(ks)                  # more energy never needs fewer dimensions
