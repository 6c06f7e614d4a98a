"""GPU parity of the adaptive-rank entry point: the rank chosen on the device by the
retained-energy count of Section 2 (sum of singular values, measured inside the sketch) against
the oracle's, and the factors against the oracle's at that rank.

The count is an integer decided by floating-point sums: both sides are given energy targets that
lie in the middle of a gap between two consecutive retained fractions of the oracle (gap at
least 1e-2), so that the decision does not hinge on rounding; what is compared is then exact.
"""
import numpy as np
import pytest
import torch

from oracle import loract_oracle as orc
from workloads import synth

from gpu_util import TOL_PARITY, check_local, ortho_tolerance, to_device, to_host

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,m,n,k_max,l,decay", [("bf16", 2048, 512, 64, 64, 0.85),
                                                      ("bf16", 1500, 384, 48, 72, 0.8),
                                                      ("f32", 600, 200, 24, 32, 0.7)])
def test_adaptive_rank_matches_oracle(dtype, m, n, k_max, l, decay):
    import paper_2509_23472_amd as L
    s = decay ** np.arange(min(m, n))
    w = synth._finish("adaptive_%dx%d" % (m, n), synth.spectrum_matrix(m, n, s, 1e-3, 11), dtype, k_max, 11)
    x64 = w.x.astype(np.float64)
    frac = orc.decompose_adaptive(x64, k_max, 1.0, seed=w.seed, l=l)[3]
    targets = []
    for j in range(1, k_max):                          # energy between fractions j-1 and j -> rank j + 1
        if frac[j] - frac[j - 1] >= 1e-2:
            targets.append((0.5 * (frac[j - 1] + frac[j]), j + 1))
    targets = targets[:: max(1, len(targets) // 4)]
    targets.append((1.0, k_max))                       # everything: capped at k_max
    assert len(targets) >= 3
    x = to_device(w.x, dtype)
    tol = TOL_PARITY[dtype] if dtype == "bf16" else 1e-4
    # rounding enters through the l-column basis and the l x n factor, before the cut to rank k: the
    # element bound is taken with their row and column norms
    ql, bl = orc.decompose(x64, l, seed=w.seed, l=l)
    un, vn = np.linalg.norm(ql, axis=1), np.linalg.norm(bl, axis=0)
    for energy, want in targets:
        print("case", w.name, dtype, "energy %.4f" % energy, "expect k", want, flush=True)
        status = torch.full((1,), -1, dtype=torch.int32, device="cuda")
        u, v, k_dev = L.loract_compress_adaptive(x, k_max, energy, l=l, seed=w.seed, status=status)
        torch.cuda.synchronize()
        k = int(k_dev.item())
        uo, vo, ko, _ = orc.decompose_adaptive(x64, k_max, energy, seed=w.seed, l=l)
        assert ko == want and k == want, (energy, k, ko, want)
        assert int(status.item()) == 0
        uh, vh = to_host(u), to_host(v)
        assert uh.shape == (m, k_max) and vh.shape == (k_max, n)
        assert np.all(uh[:, k:] == 0.0) and np.all(vh[k:, :] == 0.0)      # padded with zeros
        xo = uo @ vo
        got = uh @ vh
        assert orc.rel_fro(got, xo) <= tol
        print(check_local(got, xo, un, vn, tol, 2.0 ** -8 if dtype == "bf16" else 2.0 ** -20, "adaptive U V"))
        defect = orc.orthogonality_defect(uh[:, :k])
        assert defect <= (ortho_tolerance(w, u.dtype, uo) if dtype == "bf16" else 1e-5), defect
