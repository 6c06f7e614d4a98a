"""Helpers shared by the GPU parity tests: upload/download and the parity metrics.

Parity is judged on quantities that do not depend on the choice of basis: the reconstruction
U V (any orthonormal basis of the same range gives the same product), the orthogonality defect
of the returned U, and the approximation quality ||X - U V||.
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import loract_oracle as orc
from workloads import synth

TOL_PARITY = {"f32": 1e-5, "bf16": 2e-2}    # relative Frobenius error of Xhat, GPU vs oracle
TOL_ORTHO = 1e-3                            # ||U^T U - I||_2 on the U the GPU returns


def ortho_tolerance(w: synth.Workload, u_dtype: torch.dtype, q_oracle: np.ndarray) -> float:
    """Bound on ||U^T U - I||_2 for the returned U.

    1e-3 in general.  A U stored in bf16 carries 2^-9 relative rounding per entry, which alone
    gives a defect of order 2^-9 sqrt(k/m)-ish: above 1e-3 for the short test matrices (it is
    below 1e-3 at every benchmark shape).  There the bound is what bf16 storage of an exactly
    orthonormal basis (the oracle's Q) costs, with 50% slack.
    """
    if u_dtype != torch.bfloat16:
        return TOL_ORTHO
    stored = synth.round_to_bf16(q_oracle.astype(np.float32)).astype(np.float64)
    return max(TOL_ORTHO, 1.5 * orc.orthogonality_defect(stored))


def to_device(x32: np.ndarray, dtype: str) -> torch.Tensor:
    """Upload a float32 array whose values are representable in `dtype`."""
    if dtype == "bf16":
        bits = synth.f32_to_bf16_bits(x32)
        assert np.array_equal(synth.bf16_bits_to_f32(bits), x32), "input is not bf16-representable"
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x32, dtype=np.float32)).cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    """Download as float64 (exact widening)."""
    return t.detach().float().cpu().numpy().astype(np.float64)


def block_sumsq(a: np.ndarray, bm: int = 64, bn: int = 128) -> np.ndarray:
    """Sum of squares of every bm x bn block of `a` (ragged last blocks included)."""
    rows = np.add.reduceat(a * a, np.arange(0, a.shape[0], bm), axis=0)
    return np.add.reduceat(rows, np.arange(0, a.shape[1], bn), axis=1)


def check_local(got: np.ndarray, want: np.ndarray, un: np.ndarray, cn: np.ndarray, tol: float,
                eps: float, what: str, row_floor: float = 0.0) -> dict:
    """Local agreement of a reconstruction with the oracle's, so that a misplaced or missing
    tile cannot hide inside a global norm.

    (i)  every 64 x 128 block (the tile a workgroup of the streaming kernels owns): relative
         Frobenius error <= tol, relative to the block's own norm in the oracle (blocks whose
         oracle norm is below 1e-3 of the average block are measured against that floor);
    (ii) every element: |got - want| <= 4 eps ||u_i|| ||x_c|| + eps |want| + row_floor ||x_c||,
         where u_i is the row of U the element is formed from (oracle value; its norm does not
         depend on the choice of basis), x_c the column of X that column c of V = U^T X is the
         image of (`cn`, its norm), and eps the unit rounding of the storage type of the factors
         (2^-8 for bf16: each factor entry carries 2^-9, the stored element another 2^-9).
         Entrywise rounding of U moves v_c = U^T x_c by up to eps ||x_c|| -- not eps ||v_c||: a
         column of which the basis captures little is a cancellation -- and of V by eps ||v_c|| <=
         eps ||x_c||; by Cauchy-Schwarz the element moves by ||u_i|| times that, with a factor four
         of slack for what is not rounding (the finite accuracy of the basis).  For columns that
         the basis captures well ||v_c|| ~ ||x_c|| and nothing is given away.  `row_floor` is an
         absolute error of a row of U that does not shrink with the row: the bf16 path
         accumulates the sketch in float32, so a row of the basis is resolved to about 2^-20 of
         the typical row norm however small the row itself is (a row nearly orthogonal to the
         sampled rows is a cancellation too).  Both cancellations are met with k = 1.
    """
    d = got - want
    err = np.sqrt(block_sumsq(d))
    ref = np.sqrt(block_sumsq(want))
    floor = 1e-3 * float(ref.mean()) + 1e-300
    rel = err / np.maximum(ref, floor)
    worst = np.unravel_index(int(np.argmax(rel)), rel.shape)
    assert rel.max() <= tol, "%s: block %s relative error %.3e > %.1e" % (what, worst, rel.max(), tol)
    bound = 4.0 * eps * np.outer(un, cn) + eps * np.abs(want) + row_floor * cn[None, :] + 1e-300
    ratio = np.abs(d) / bound
    at = np.unravel_index(int(np.argmax(ratio)), ratio.shape)
    assert ratio.max() <= 1.0, "%s: element %s off by %.3e, bound %.3e" % (what, at, abs(d[at]), bound[at])
    return {"block_max": float(rel.max()), "elem_max_over_bound": float(ratio.max())}


def sample_row_blocks(m: int, every: int, bm: int = 64) -> np.ndarray:
    """Row ids of every `every`-th block of `bm` rows, plus the last block (ragged tail included)."""
    nblk = (m + bm - 1) // bm
    blocks = sorted(set(range(0, nblk, every)) | {nblk - 1})
    return np.concatenate([np.arange(b * bm, min(m, (b + 1) * bm)) for b in blocks])


def check_compress_parity(w: synth.Workload, u_gpu: torch.Tensor, v_gpu: torch.Tensor,
                          xhat_gpu: torch.Tensor = None, t: int = 0, idx=None,
                          tol: float = None, oracle_factors=None, strict_ortho: bool = False,
                          local: bool = True, rows: np.ndarray = None):
    """Compare GPU factors (and optionally the GPU reconstruction) with the oracle; returns a dict.

    Checked: the global relative Frobenius error of U V (and of the GPU's own reconstruction)
    against the oracle's, the same per 64 x 128 block and per element (`check_local`), the
    orthogonality defect of the returned U, and the approximation quality ||X - U V|| / ||X||
    against the oracle's (within 10% plus what storing the oracle's own factors in the factor
    type costs).

    `rows` (whole blocks of 64 rows, see `sample_row_blocks`) restricts the comparisons of the
    m x n products to those rows, each of which the oracle computes exactly as it would in the
    full comparison (a row of U V needs that row of U only): for the largest sites, where forming
    and comparing the whole m x n product several times over would take minutes.  The
    factorisation itself is always the full one, and U is always checked whole.
    """
    tol = TOL_PARITY[w.dtype] if tol is None else tol
    x = w.x.astype(np.float64) if rows is None else w.x[rows].astype(np.float64)
    if oracle_factors is None:
        oracle_factors = orc.decompose(w.x.astype(np.float64), w.k, t=t, seed=w.seed, idx=idx)
    uo, vo = oracle_factors
    u, v = to_host(u_gpu), to_host(v_gpu)
    assert u.shape == (w.m, w.k) and v.shape == (w.k, w.n)
    assert np.all(np.isfinite(u)) and np.all(np.isfinite(v))
    ortho = orc.orthogonality_defect(u)
    uo_r, u_r = (uo, u) if rows is None else (uo[rows], u[rows])
    xo = orc.reconstruct(uo_r, vo)
    rebuilt = u_r @ v
    res = {
        "parity_factors": orc.rel_fro(rebuilt, xo),
        "ortho": ortho,
        "quality_gpu": orc.rel_fro(rebuilt, x),
        "quality_oracle": orc.rel_fro(xo, x),
    }
    assert res["parity_factors"] <= tol, res
    res["ortho_tol"] = TOL_ORTHO if strict_ortho else ortho_tolerance(w, u_gpu.dtype, uo)
    assert res["ortho"] <= res["ortho_tol"], res
    # approximation quality: a basis-independent scalar that is far below the parity tolerance
    bf16_factors = u_gpu.dtype == torch.bfloat16
    # (bf16 inputs: the basis enters the projection rounded to bf16 whatever the factor type is)
    storage_noise = 0.0
    if w.dtype == "bf16":
        ub = synth.round_to_bf16(uo.astype(np.float32)).astype(np.float64)
        vb = ub.T @ w.x.astype(np.float64)
        if bf16_factors:
            vb = synth.round_to_bf16(vb.astype(np.float32)).astype(np.float64)
        u_used = ub if bf16_factors else uo
        storage_noise = abs(orc.rel_fro((u_used if rows is None else u_used[rows]) @ vb, x) - res["quality_oracle"])
        del ub, vb, u_used
    res["quality_tol"] = 0.1 * res["quality_oracle"] + 1.5 * storage_noise + 1e-6
    assert abs(res["quality_gpu"] - res["quality_oracle"]) <= res["quality_tol"], res
    if local:
        # bf16 inputs: the basis enters the projection rounded to bf16 whatever type the factors
        # are returned in, so the unit rounding of the comparison is that of bf16 storage
        eps = 2.0 ** -8 if (bf16_factors or w.dtype == "bf16") else 2.0 ** -20
        un = np.linalg.norm(uo_r, axis=1)
        cn = np.sqrt(np.einsum("ij,ij->j", w.x, w.x, dtype=np.float64))     # column norms of X
        # float32 accumulation of the sketch: absolute resolution of a row of the basis
        row_floor = 2.0 ** -20 * float(np.sqrt(np.mean(un * un))) if w.dtype == "bf16" else 0.0
        loc = check_local(rebuilt, xo, un, cn, tol, eps, "U V rebuilt on the host", row_floor)
        res["block_max_factors"], res["elem_factors"] = loc["block_max"], loc["elem_max_over_bound"]
    del rebuilt
    if xhat_gpu is not None:
        xh = to_host(xhat_gpu if rows is None else xhat_gpu[torch.from_numpy(rows).to(xhat_gpu.device)])
        res["parity_reconstruct"] = orc.rel_fro(xh, xo)
        assert res["parity_reconstruct"] <= tol, res
        if local:
            eps_out = eps if xhat_gpu.dtype != torch.bfloat16 else max(eps, 2.0 ** -8)
            loc = check_local(xh, xo, un, cn, tol, eps_out, "GPU reconstruction", row_floor)
            res["block_max_reconstruct"], res["elem_reconstruct"] = loc["block_max"], loc["elem_max_over_bound"]
    return res
