"""GPU parity: the HIP library (through its C ABI binding) against the fp64 CPU oracle on the
same seeded inputs and the same seed-derived sample indices.

Tolerances (relative Frobenius error of the reconstruction, GPU vs oracle): 1e-5 for fp32
inputs, 2e-2 for bf16 inputs; ||U^T U - I||_2 <= 1e-3 on the returned U.
"""
import numpy as np
import pytest
import torch

from oracle import loract_oracle as orc
from workloads import synth

from gpu_util import TOL_PARITY, check_compress_parity, to_device, to_host

pytestmark = pytest.mark.gpu


def _lib():
    import paper_2509_23472_amd as L
    return L


def _spectrum_workload(m, n, k, seed, dtype="bf16", decay=0.9, noise=1e-3):
    s = decay ** np.arange(min(m, n))
    x = synth.spectrum_matrix(m, n, s, noise, seed)
    return synth._finish("spec_%dx%d_k%d" % (m, n, k), x, dtype, k, seed)


def _run(w, t=0, factor_dtype=None, idx=None):
    L = _lib()
    print("case", w.name, "dtype", w.dtype, "k", w.k, "t", t, flush=True)
    x = to_device(w.x, w.dtype)
    status = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    u, v = L.loract_compress(x, w.k, t=t, seed=w.seed, idx=idx, factor_dtype=factor_dtype,
                             status=status)
    xhat = L.loract_reconstruct(u, v)
    torch.cuda.synchronize()
    return x, u, v, xhat, int(status.item())


def _strict_ortho_with_fp32_factors(w, oracle_factors):
    """The same matrix with fp32 factors: what the orthonormalisation itself leaves, before any
    bf16 storage rounding of U, must meet the 1e-3 bound with nothing relaxed."""
    x, u, v, xhat, status = _run(w, factor_dtype=torch.float32)
    res = check_compress_parity(w, u, v, xhat, oracle_factors=oracle_factors, strict_ortho=True)
    print("fp32 factors:", res)
    assert res["ortho"] <= 1e-3


# ----------------------------------------------------------------------------- config 1 (fp32)


def test_c1_fp32_lowrank_full_size():
    w = synth.c1_lowrank_f32()
    x, u, v, xhat, status = _run(w)
    res = check_compress_parity(w, u, v, xhat)
    print(res)
    assert status == 0
    assert u.dtype == torch.float32 and v.dtype == torch.float32
    assert res["ortho"] <= 1e-5
    # the signal has rank exactly k, so the approximation error is at the noise level
    assert res["quality_gpu"] <= 1e-3


@pytest.mark.parametrize("m,n,k", [(16, 16, 16), (70, 33, 1), (257, 130, 19), (300, 70, 64),
                                    (129, 300, 65)])
def test_fp32_small_and_ragged_shapes(m, n, k):
    w = _spectrum_workload(m, n, k, seed=m + n + k, dtype="f32", decay=0.8, noise=1e-4)
    x, u, v, xhat, status = _run(w)
    print(check_compress_parity(w, u, v, xhat))


def test_fp32_exact_rank_is_recovered():
    # proof of Theorem 4.2, first case: rank(X) <= k  =>  U V = X (here to fp32 accuracy)
    w = synth.exact_rank(200, 96, 8, seed=5, dtype="f32")
    x, u, v, xhat, status = _run(w)
    assert orc.rel_fro(to_host(xhat), w.x.astype(np.float64)) <= 1e-5
    print(check_compress_parity(w, u, v, xhat))


# ----------------------------------------------------------------------------- bf16, small and ragged


@pytest.mark.parametrize("m,n,k", [(64, 64, 8), (333, 200, 24), (1000, 520, 70), (130, 203, 17),
                                    (2050, 96, 96), (97, 1031, 33), (515, 264, 130), (1795, 410, 1)])
def test_bf16_small_and_ragged_shapes(m, n, k):
    # (rank 1: U is the normalised sketch column itself, so rows nearly orthogonal to the sampled
    # row show the float32 accumulation of the sketch undiluted)
    w = _spectrum_workload(m, n, k, seed=3 * m + n + k, dtype="bf16")
    x, u, v, xhat, status = _run(w)
    of = orc.decompose(w.x.astype(np.float64), w.k, seed=w.seed)
    print(check_compress_parity(w, u, v, xhat, oracle_factors=of))
    assert u.dtype == torch.bfloat16 and v.dtype == torch.bfloat16
    _strict_ortho_with_fp32_factors(w, of)


@pytest.mark.parametrize("m,n,k", [(130, 64, 17), (1000, 512, 72), (4100, 1024, 136), (520, 640, 264),
                                    (777, 320, 320), (129, 128, 128), (2048, 192, 8), (385, 448, 200),
                                    (1500, 512, 250), (600, 256, 16), (700, 256, 33), (602, 1024, 1)])
def test_bf16_streaming_kernels_ragged_rows_and_all_rank_tiles(m, n, k):
    # n % 64 == 0 selects the matrix-core streaming kernels; the shapes walk through every
    # accumulator-tile variant (kp <= 64, <= 128, <= 256, two column blocks), the maximum rank,
    # row counts that end inside a 128-row tile, and K ranges that do not divide evenly; for the
    # Cholesky kernels: one panel only (16), padding inside the last panel (33, 72, 136, 250), both
    # register-resident sizes (<= 128, <= 256) and the in-place kernel above them (264, 320).
    w = _spectrum_workload(m, n, k, seed=7 * m + n + k, dtype="bf16", decay=0.93)
    x, u, v, xhat, status = _run(w)
    of = orc.decompose(w.x.astype(np.float64), w.k, seed=w.seed)
    print(check_compress_parity(w, u, v, xhat, oracle_factors=of))
    _strict_ortho_with_fp32_factors(w, of)


def test_bf16_streaming_kernels_with_row_pitch_and_power_iteration():
    L = _lib()
    w = _spectrum_workload(900, 256, 40, seed=77, dtype="bf16")
    big = torch.zeros((900, 320), dtype=torch.bfloat16, device="cuda")
    big[:, :256] = to_device(w.x, "bf16")
    u, v = L.loract_compress(big[:, :256], w.k, t=1, seed=w.seed)
    out_big = torch.full((900, 384), -3.0, dtype=torch.bfloat16, device="cuda")
    L.loract_reconstruct(u, v, out=out_big[:, :256])
    torch.cuda.synchronize()
    print(check_compress_parity(w, u, v, out_big[:, :256], t=1))
    assert torch.all(out_big[:, 256:] == -3.0)


def test_bf16_input_with_fp32_factors():
    w = _spectrum_workload(700, 256, 40, seed=9, dtype="bf16")
    x, u, v, xhat, status = _run(w, factor_dtype=torch.float32)
    res = check_compress_parity(w, u, v, xhat)
    print(res)
    assert u.dtype == torch.float32
    assert res["ortho"] <= 1e-5          # fp32 U is orthonormal to working precision


def test_bf16_exact_rank_is_recovered():
    w = synth.exact_rank(512, 128, 8, seed=6, dtype="bf16")
    x, u, v, xhat, status = _run(w)
    # bf16 factors carry 2^-9 relative rounding each
    assert orc.rel_fro(to_host(xhat), w.x.astype(np.float64)) <= 1e-2
    print(check_compress_parity(w, u, v, xhat))


def test_row_stride_larger_than_n():
    L = _lib()
    w = _spectrum_workload(300, 120, 20, seed=4, dtype="bf16")
    big = torch.zeros((300, 160), dtype=torch.bfloat16, device="cuda")
    big[:, :120] = to_device(w.x, "bf16")
    xv = big[:, :120]
    u, v = L.loract_compress(xv, w.k, seed=w.seed)
    out_big = torch.full((300, 200), 7.0, dtype=torch.bfloat16, device="cuda")
    L.loract_reconstruct(u, v, out=out_big[:, :120])
    torch.cuda.synchronize()
    print(check_compress_parity(w, u, v, out_big[:, :120]))
    assert torch.all(out_big[:, 120:] == 7.0)      # nothing written outside the view


def test_explicit_indices_equal_seed_derived_and_runs_are_deterministic():
    L = _lib()
    w = _spectrum_workload(900, 256, 48, seed=21, dtype="bf16")
    x = to_device(w.x, "bf16")
    idx = orc.sample_indices(w.m, w.k, w.seed).tolist()
    assert idx == L.loract_sample_indices(w.m, w.k, w.seed)
    u1, v1 = L.loract_compress(x, w.k, seed=w.seed)
    u1, v1 = u1.clone(), v1.clone()
    u2, v2 = L.loract_compress(x, w.k, seed=999, idx=idx)
    u2, v2 = u2.clone(), v2.clone()
    u3, v3 = L.loract_compress(x, w.k, seed=w.seed)
    torch.cuda.synchronize()
    assert torch.equal(u1, u2) and torch.equal(v1, v2)      # bit-identical
    assert torch.equal(u1, u3) and torch.equal(v1, v3)


def test_power_iterations_match_oracle():
    # the power rounds of Algorithm 1 with t = 1 and 2
    for t in (1, 2):
        w = _spectrum_workload(600, 256, 24, seed=30 + t, dtype="f32", decay=0.85, noise=1e-4)
        x, u, v, xhat, status = _run(w, t=t)
        print(t, check_compress_parity(w, u, v, xhat, t=t, tol=1e-4))
    w = _spectrum_workload(800, 320, 32, seed=33, dtype="bf16")
    x, u, v, xhat, status = _run(w, t=1)
    print(check_compress_parity(w, u, v, xhat, t=1))


def _check_degenerate(L, xs, idx, idx_independent, k, expect_dropped):
    x = to_device(xs, "bf16")
    status = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    u, v = L.loract_compress(x, k, idx=idx, status=status)
    torch.cuda.synchronize()
    flagged = bool(int(status.item()) & L.STATUS_RANK_DEFICIENT)
    uh, vh = to_host(u), to_host(v)
    assert np.all(np.isfinite(uh)) and np.all(np.isfinite(vh))
    gram = uh.T @ uh
    d = np.diag(gram)
    dropped = d == 0.0
    print("flagged", flagged, "diag of U^T U:", np.round(d, 4))
    # the flag is raised exactly when a direction was dropped (a zero column of U) ...
    assert flagged == bool(dropped.any())
    if expect_dropped is not None:
        assert int(dropped.sum()) == expect_dropped
    # ... the remaining columns are orthonormal (up to bf16 storage of a short matrix) ...
    keep = ~dropped
    assert np.linalg.norm(gram[np.ix_(keep, keep)] - np.eye(keep.sum()), 2) <= 3e-3
    # ... and the product still contains the projection onto range(Y).  Only that part is
    # unique (the completion direction is arbitrary, for the oracle's QR as well), so compare
    # it with the oracle run on the independent sampled rows alone, and require that the extra
    # direction, if any, does not make the approximation worse.
    x64 = xs.astype(np.float64)
    uo, vo = orc.decompose(x64, len(idx_independent), idx=idx_independent)
    xo = orc.reconstruct(uo, vo)
    got = uh @ vh
    assert orc.rel_fro(uo @ (uo.T @ got), xo) <= TOL_PARITY["bf16"]
    assert np.linalg.norm(x64 - got) <= np.linalg.norm(x64 - xo) * (1 + TOL_PARITY["bf16"])


def test_duplicate_sampled_rows_stay_finite_and_accurate():
    # Padding tokens give identical rows; sampling two of them makes the sketch exactly rank
    # deficient.  The dependent direction is either dropped (flag + zero column) or replaced by
    # an arbitrary orthonormal completion; both leave U V the projection of X onto range(Y).
    L = _lib()
    w = _spectrum_workload(400, 128, 12, seed=8, dtype="bf16")
    xs = w.x.copy()
    xs[7, :] = xs[3, :]
    idx = sorted(set([3, 7] + orc.sample_indices(400, 12, 1).tolist()))[:12]
    _check_degenerate(L, xs, idx, [i for i in idx if i != 7], 12, None)


def test_all_zero_sampled_row_is_dropped_and_flagged():
    # A sampled row of zeros gives an exactly zero sketch column: that direction must be
    # dropped (zero column of U) and LORACT_STATUS_RANK_DEFICIENT raised.
    L = _lib()
    w = _spectrum_workload(400, 128, 12, seed=18, dtype="bf16")
    xs = w.x.copy()
    xs[5, :] = 0.0
    idx = sorted(set([5] + orc.sample_indices(400, 12, 2).tolist()))[:12]
    _check_degenerate(L, xs, idx, [i for i in idx if i != 5], 12, 1)


# ----------------------------------------------------------------------------- consumers of the factors


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_reconstruct_alone_on_given_factors(dtype):
    L = _lib()
    rng = np.random.default_rng(1)
    m, n, k = 391, 277, 37
    u = rng.standard_normal((m, k)).astype(np.float32)
    v = rng.standard_normal((k, n)).astype(np.float32)
    if dtype == "bf16":
        u, v = synth.round_to_bf16(u), synth.round_to_bf16(v)
    ref = orc.reconstruct(u, v)
    out = L.loract_reconstruct(to_device(u, dtype), to_device(v, dtype))
    out32 = L.loract_reconstruct(to_device(u, dtype), to_device(v, dtype), out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert orc.rel_fro(to_host(out32), ref) <= 1e-6
    assert orc.rel_fro(to_host(out), ref) <= (3e-3 if dtype == "bf16" else 1e-6)


@pytest.mark.parametrize("dtype,m,n,k,n_out,r", [("bf16", 777, 256, 32, 320, 16),
                                                  ("bf16", 300, 136, 20, 75, 5),
                                                  ("f32", 260, 96, 12, 130, 8),
                                                  # matrix-core path with several 64-column tiles of U
                                                  # and many row shares, ragged rows, wide LoRA rank
                                                  ("bf16", 4100, 512, 256, 384, 16),
                                                  ("bf16", 9000, 320, 136, 256, 64),
                                                  ("bf16", 2111, 256, 72, 128, 33)])
def test_lora_grad_matches_oracle(dtype, m, n, k, n_out, r):
    L = _lib()
    w = _spectrum_workload(m, n, k, seed=m + r, dtype=dtype)
    rng = np.random.default_rng(m)
    dy = rng.standard_normal((m, n_out)).astype(np.float32)
    b = (rng.standard_normal((r, n_out)) / np.sqrt(r)).astype(np.float32)
    if dtype == "bf16":
        dy, b = synth.round_to_bf16(dy), synth.round_to_bf16(b)
    x = to_device(w.x, dtype)
    u, v = L.loract_compress(x, k, seed=w.seed)
    g = L.loract_lora_grad(u, v, to_device(dy, dtype), to_device(b, dtype), scale=0.5)
    torch.cuda.synchronize()
    # (a) the contraction itself, on the factors the GPU produced: tight
    ref_same_factors = orc.lora_grad(to_host(u), to_host(v), dy, b, 0.5)
    assert orc.rel_fro(to_host(g), ref_same_factors) <= (1e-5 if dtype == "f32" else 1e-4)
    # (b) end to end against the oracle's own factors: the path tolerance
    uo, vo = orc.decompose(w.x.astype(np.float64), k, seed=w.seed)
    ref = orc.lora_grad(uo, vo, dy, b, 0.5)
    assert orc.rel_fro(to_host(g), ref) <= TOL_PARITY[dtype]


def test_gaussian_generator_matches_oracle_definition():
    L = _lib()
    l, n, seed = 9, 517, 77
    ref = orc.gaussian_omega_t(l, n, seed)
    g32 = L.loract_gaussian_omega_t(l, n, torch.float32, seed)
    g16 = L.loract_gaussian_omega_t(l, n, torch.bfloat16, seed)
    torch.cuda.synchronize()
    assert np.max(np.abs(to_host(g32) - ref)) <= 1e-6
    assert np.max(np.abs(to_host(g16) - ref) / (np.abs(ref) + 1e-3)) <= 2.0 ** -8


# ----------------------------------------------------------------------------- RSVD comparator


@pytest.mark.parametrize("dtype,m,n,k,oversample,iters", [
    ("f32", 300, 128, 12, 0, 0), ("f32", 300, 128, 12, 5, 1),
    ("bf16", 640, 256, 24, 0, 0), ("bf16", 640, 256, 24, 8, 0), ("bf16", 700, 320, 40, 8, 1),
])
def test_rsvd_comparator_matches_oracle(dtype, m, n, k, oversample, iters):
    # Section 3.2's comparator, with the Gaussian test matrix handed to both sides as data.
    L = _lib()
    w = _spectrum_workload(m, n, k, seed=5 * m + k + oversample, dtype=dtype, decay=0.85)
    l = k + oversample
    omega_t = synth.gaussian_test_matrix(l, n, seed=77 + oversample).astype(np.float32)
    if dtype == "bf16":
        omega_t = synth.round_to_bf16(omega_t)
    x = to_device(w.x, dtype)
    status = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    u, v = L.loract_rsvd(x, k, oversample=oversample, power_iters=iters,
                         omega_t=to_device(omega_t, dtype), status=status)
    torch.cuda.synchronize()
    uo, vo = orc.rsvd(w.x.astype(np.float64), k, oversample=oversample, power_iters=iters,
                      omega_t=omega_t.astype(np.float64))
    res = check_compress_parity(w, u, v, oracle_factors=(uo, vo),
                                tol=1e-4 if dtype == "f32" else None)
    print(res, "status", int(status.item()))
    assert int(status.item()) == 0


def test_rsvd_with_device_generated_test_matrix():
    # seed-derived Gaussian test matrix: both sides implement the same counter-based generator
    L = _lib()
    w = _spectrum_workload(512, 192, 16, seed=91, dtype="bf16", decay=0.8)
    x = to_device(w.x, "bf16")
    u, v = L.loract_rsvd(x, 16, oversample=4, power_iters=0, seed=1234)
    torch.cuda.synchronize()
    omega_t = synth.round_to_bf16(orc.gaussian_omega_t(20, 192, 1234).astype(np.float32))
    uo, vo = orc.rsvd(w.x.astype(np.float64), 16, oversample=4, omega_t=omega_t.astype(np.float64))
    print(check_compress_parity(w, u, v, oracle_factors=(uo, vo)))


@pytest.mark.parametrize("dtype,m,n,k,l,t", [("f32", 500, 130, 8, 13, 0), ("bf16", 2100, 512, 32, 48, 0),
                                             ("bf16", 1031, 256, 16, 40, 1), ("bf16", 4096, 1024, 64, 96, 0)])
def test_oversampled_row_sample_truncated_to_rank_k(dtype, m, n, k, l, t):
    # Theorem 4.3's setting: l > k sampled rows, factors cut to the k leading singular triplets
    L = _lib()
    w = _spectrum_workload(m, n, k, seed=3 * m + l, dtype=dtype, decay=0.9)
    x = to_device(w.x, dtype)
    status = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    u, v = L.loract_compress(x, k, t=t, seed=w.seed, l=l, status=status)
    xhat = L.loract_reconstruct(u, v)
    torch.cuda.synchronize()
    uo, vo = orc.decompose(w.x.astype(np.float64), k, t=t, seed=w.seed, l=l)
    res = check_compress_parity(w, u, v, xhat, oracle_factors=(uo, vo),
                                tol=1e-4 if dtype == "f32" else None)
    print(res, "status", int(status.item()))
    assert int(status.item()) == 0
    # the extra sampled rows must not hurt: same matrix, l = k
    u0, v0 = L.loract_compress(x, k, t=t, seed=w.seed)
    torch.cuda.synchronize()
    e_k = orc.rel_fro(to_host(u0) @ to_host(v0), w.x.astype(np.float64))
    print("quality l=k %.4e  l=%d %.4e" % (e_k, l, res["quality_gpu"]))


def test_oversampled_explicit_indices():
    L = _lib()
    w = _spectrum_workload(700, 192, 12, seed=17, dtype="bf16", decay=0.85)
    idx = sorted(np.random.default_rng(3).choice(700, size=20, replace=False).tolist())
    x = to_device(w.x, "bf16")
    u, v = L.loract_compress(x, 12, idx=idx, l=20)
    torch.cuda.synchronize()
    uo, vo = orc.decompose(w.x.astype(np.float64), 12, idx=idx, l=20)
    print(check_compress_parity(w, u, v, oracle_factors=(uo, vo)))
    with pytest.raises(Exception):
        L.loract_compress(x, 12, idx=idx[:12], l=20)


@pytest.mark.parametrize("power,factor", [(1.8, "bf16"), (2.0, "f32"), (2.6, "bf16")])
def test_tall_ill_conditioned_sketch_uses_the_higher_order_finish(power, factor):
    # Tall matrix (the degree-4 finish of round 2 is prepared from 32768 rows on) whose sketch has a
    # condition number of 1e6..1e9: round 1 leaves ||Q1^T Q1 - I|| between the reach of the
    # first-order correction and far beyond the reach of the series, so the three exits that do work
    # on Q1 (first order, degree 4, second factorisation) are all exercised.  Whatever the exit, the
    # result must be orthonormal and match the oracle.
    L = _lib()
    m, n, k = 32768, 256, 64
    s = np.arange(1, n + 1, dtype=np.float64) ** -power
    w = synth._finish("tall_%g" % power, synth.spectrum_matrix(m, n, s, 1e-4, 77), "bf16", k, 77)
    x = to_device(w.x, "bf16")
    status = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    fd = torch.float32 if factor == "f32" else None
    print("case", w.name, "factor", factor, flush=True)
    u, v = L.loract_compress(x, k, seed=w.seed, factor_dtype=fd, status=status)
    xhat = L.loract_reconstruct(u, v)
    torch.cuda.synchronize()
    res = check_compress_parity(w, u, v, xhat, strict_ortho=True)
    print(power, factor, res, "status", int(status.item()))
    if factor == "f32":
        assert res["ortho"] <= 3e-4      # no bf16 rounding of U: what the finish itself leaves
