"""GPU parity of the pre-norm unit (Section 3.3, Eqs. 6-10) against the fp64 oracle: the two row
kernels on their own, and the whole chain norm -> compress -> reconstruct -> backward."""
import numpy as np
import pytest
import torch

from oracle import loract_oracle as orc
from workloads import synth

from gpu_util import TOL_PARITY, to_device, to_host

pytestmark = pytest.mark.gpu


def _inputs(m, n, dtype, seed):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((m, n)) * rng.uniform(0.5, 3.0, size=(m, 1))).astype(np.float32)
    gamma = rng.uniform(0.5, 1.5, size=n).astype(np.float32)
    grad_a = rng.standard_normal((m, n)).astype(np.float32)
    if dtype == "bf16":
        x, grad_a = synth.round_to_bf16(x), synth.round_to_bf16(grad_a)
    return x, gamma, grad_a


@pytest.mark.parametrize("dtype,m,n", [("bf16", 257, 512), ("bf16", 130, 1032), ("bf16", 64, 203),
                                        ("f32", 100, 96), ("f32", 33, 77), ("bf16", 5, 11008)])
def test_prenorm_forward_and_backward_kernels(dtype, m, n):
    import paper_2509_23472_amd as L
    x, gamma, grad_a = _inputs(m, n, dtype, seed=m + n)
    g_dev = torch.from_numpy(gamma).cuda()
    a_gpu, rms_gpu = L.loract_prenorm_forward(to_device(x, dtype), g_dev)
    torch.cuda.synchronize()
    a_ref, rms_ref = orc.prenorm_forward(x, gamma)
    tol = 1e-5 if dtype == "f32" else 4e-3            # one bf16 rounding of the output
    assert np.max(np.abs(to_host(rms_gpu) - rms_ref) / rms_ref) <= 1e-5
    assert orc.rel_fro(to_host(a_gpu), a_ref) <= tol
    # backward on the A the GPU itself stored (so both sides start from identical inputs)
    a_in = to_host(a_gpu)
    dx_gpu = L.loract_prenorm_backward(a_gpu, rms_gpu, g_dev, to_device(grad_a, dtype))
    torch.cuda.synchronize()
    dx_ref = orc.prenorm_backward(a_in, to_host(rms_gpu), gamma, grad_a)
    assert orc.rel_fro(to_host(dx_gpu), dx_ref) <= tol


def test_prenorm_chain_through_compression():
    # forward: A = Norm(X), compress A (Algorithm 1), keep U, V and the RMS vector;
    # backward: A~ = U V, then Eqs. (8)-(10).  Compared with the same chain in the oracle.
    import paper_2509_23472_amd as L
    m, n, k = 1024, 512, 48
    s = 0.9 ** np.arange(n)
    x = synth.round_to_bf16(synth.spectrum_matrix(m, n, s, 1e-3, seed=5).astype(np.float32))
    rng = np.random.default_rng(6)
    gamma = rng.uniform(0.5, 1.5, size=n).astype(np.float32)
    grad_a = synth.round_to_bf16(rng.standard_normal((m, n)).astype(np.float32))
    g_dev = torch.from_numpy(gamma).cuda()
    a_gpu, rms_gpu = L.loract_prenorm_forward(to_device(x, "bf16"), g_dev)
    u, v = L.loract_compress(a_gpu, k, seed=11)
    a_tilde = L.loract_reconstruct(u, v)
    dx_gpu = L.loract_prenorm_backward(a_tilde, rms_gpu, g_dev, to_device(grad_a, "bf16"))
    torch.cuda.synchronize()
    # oracle chain, starting from the bf16 A the GPU stored (the matrix Algorithm 1 is given)
    a_in = to_host(a_gpu)
    uo, vo = orc.decompose(a_in, k, seed=11)
    dx_ref = orc.prenorm_backward(orc.reconstruct(uo, vo), to_host(rms_gpu), gamma, grad_a)
    err = orc.rel_fro(to_host(dx_gpu), dx_ref)
    print("pre-norm chain parity", err)
    assert err <= TOL_PARITY["bf16"]
