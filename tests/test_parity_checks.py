"""The GPU parity helper itself, exercised on the CPU: an emulated bf16 result (the oracle's
factors stored in bf16) must pass, and a planted mistake -- a misplaced tile, one wrong element,
a basis that spans part of a wrong subspace -- must be rejected even where the global
Frobenius tolerance alone would let it through.
"""
import numpy as np
import pytest
import torch

from oracle import loract_oracle as orc
from workloads import synth

from gpu_util import check_compress_parity


def _emulated(m, n, k, seed, power=1.5):
    s = np.arange(1, min(m, n) + 1, dtype=np.float64) ** -power
    w = synth._finish("emu", synth.spectrum_matrix(m, n, s, 1e-3, seed), "bf16", k, seed)
    x = w.x.astype(np.float64)
    uo, vo = orc.decompose(x, k, seed=seed)
    ub = torch.from_numpy(uo.astype(np.float32)).bfloat16()
    vb = (ub.double().T @ torch.from_numpy(x)).float().bfloat16()
    xh = (ub.double() @ vb.double()).float().bfloat16()
    return w, (uo, vo), ub, vb, xh


def test_emulated_bf16_result_passes_and_planted_mistakes_fail():
    w, of, ub, vb, xh = _emulated(2048, 1024, 64, 11)
    res = check_compress_parity(w, ub, vb, xh, oracle_factors=of)
    assert res["block_max_reconstruct"] < 5e-3 and res["elem_reconstruct"] < 0.5
    # a 64 x 128 tile written to the wrong place: 1/256 of the matrix, invisible to the global norm
    bad = xh.clone()
    bad[128:192, 256:384] = xh[0:64, 0:128]
    assert orc.rel_fro(bad.double().numpy(), orc.reconstruct(*of)) < 2e-1
    with pytest.raises(AssertionError, match="block"):
        check_compress_parity(w, ub, vb, bad, oracle_factors=of)
    # one wrong element
    bad = xh.clone()
    bad[77, 300] += 0.25
    with pytest.raises(AssertionError, match="element"):
        check_compress_parity(w, ub, vb, bad, oracle_factors=of)
    # a tile of V left unwritten (zeros)
    badv = vb.clone()
    badv[:, 512:640] = 0
    with pytest.raises(AssertionError):
        check_compress_parity(w, ub, badv, None, oracle_factors=of)


def test_wrong_trailing_subspace_is_rejected_by_the_quality_check():
    # an orthonormal U whose trailing half spans random directions: U V stays within the global
    # parity tolerance of a matrix with a steep spectrum, the approximation quality does not
    w, of, ub, vb, xh = _emulated(1536, 768, 64, 5, power=1.5)
    x = w.x.astype(np.float64)
    uo = of[0].copy()
    rng = np.random.default_rng(0)
    uo[:, 32:] = rng.standard_normal((w.m, 32))
    q, _ = np.linalg.qr(uo)
    ub2 = torch.from_numpy(q.astype(np.float32)).bfloat16()
    vb2 = (ub2.double().T @ torch.from_numpy(x)).float().bfloat16()
    with pytest.raises(AssertionError):
        check_compress_parity(w, ub2, vb2, None, oracle_factors=of)
