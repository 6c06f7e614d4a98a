"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times.  The fp64 oracle finishes each of these in seconds, so the whole reconstruction
is compared (not a sample).  Inputs are the seeded synthetic stand-ins for the paper's
ViT-B/16 and LLaMA2-7B activations (workloads/synth.py).
"""
import time

import numpy as np
import pytest
import torch

from oracle import loract_oracle as orc
from workloads import synth

from gpu_util import TOL_PARITY, check_compress_parity, sample_row_blocks, to_device, to_host

pytestmark = pytest.mark.gpu


def _compress_reconstruct(w):
    import paper_2509_23472_amd as L
    print("case", w.name, "bytes", w.nbytes, flush=True)
    x = to_device(w.x, w.dtype)
    status = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    u, v = L.loract_compress(x, w.k, seed=w.seed, status=status)
    xhat = L.loract_reconstruct(u, v)
    torch.cuda.synchronize()
    return L, x, u, v, xhat, int(status.item())


@pytest.mark.parametrize("name", ["c2a", "c2b"])
def test_c2_vit_sites(name):
    w = synth.FULL_SIZE[name]()
    L, x, u, v, xhat, status = _compress_reconstruct(w)
    res = check_compress_parity(w, u, v, xhat, strict_ortho=True)
    print(name, res, "status", status)
    assert status == 0


def test_c3_llama_prenorm_site_with_lora_grad():
    w = synth.c3_llama()
    L, x, u, v, xhat, status = _compress_reconstruct(w)
    t0 = time.time()
    uo, vo = orc.decompose(w.x.astype(np.float64), w.k, seed=w.seed)
    print("oracle decompose %.1fs" % (time.time() - t0), flush=True)
    res = check_compress_parity(w, u, v, xhat, oracle_factors=(uo, vo), strict_ortho=True)
    print("c3", res, "status", status)
    assert status == 0
    dy, b = w.extras["dY"], w.extras["B_lora"]
    g = L.loract_lora_grad(u, v, to_device(dy, "bf16"), to_device(b, "bf16"), scale=w.extras["scale"])
    torch.cuda.synchronize()
    ref = orc.lora_grad(uo, vo, dy, b, w.extras["scale"])
    err = orc.rel_fro(to_host(g), ref)
    print("c3 lora_grad parity", err)
    assert g.shape == (w.n, w.extras["r_lora"])
    assert err <= TOL_PARITY["bf16"]


def test_c4_llama_mlp_site():
    w = synth.c4_mlp()
    L, x, u, v, xhat, status = _compress_reconstruct(w)
    res = check_compress_parity(w, u, v, xhat, strict_ortho=True)
    print("c4", res, "status", status)
    assert status == 0


def test_c5_long_context_site():
    # one 65536 x 4096 site of the long-context stream (layer 0, site 0), k = 256
    w = synth.c5_long_context_site(0, 0)
    L, x, u, v, xhat, status = _compress_reconstruct(w)
    t0 = time.time()
    uo, vo = orc.decompose(w.x.astype(np.float64), w.k, seed=w.seed)
    print("oracle decompose %.1fs" % (time.time() - t0), flush=True)
    # (the m x n products on every 16th block of 64 rows, each row exact; U on all of its rows)
    res = check_compress_parity(w, u, v, xhat, oracle_factors=(uo, vo), strict_ortho=True,
                                rows=sample_row_blocks(w.m, 16))
    print("c5", res, "status", status)
    assert status == 0


@pytest.mark.parametrize("layer,site", [(0, 0), (0, 1), (0, 2), (0, 3), (0, 4), (0, 5), (0, 6),
                                        (13, 3), (31, 5)])
def test_c5_stream_sites_generated_on_the_gpu(layer, site):
    # The sites of the long-context stream as bench.py streams them: generated on the GPU by the
    # shared harness generator, compressed there, and the very same bits downloaded for the oracle.
    # All seven sites of layer 0 (site 6 is the 65536 x 11008 down-projection input) and one site
    # of two other layers.
    import paper_2509_23472_amd as L
    from workloads import gpu_sites
    xg = gpu_sites.c5_site_on_gpu(torch, layer, site)
    torch.cuda.synchronize()
    m, n, k = xg.shape[0], xg.shape[1], gpu_sites.C5_RANK
    seed = gpu_sites.c5_site_seed(layer, site)
    print("case c5 stream layer", layer, "site", site, "shape", (m, n), flush=True)
    status = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    u, v = L.loract_compress(xg, k, seed=seed, status=status)
    xhat = L.loract_reconstruct(u, v)
    torch.cuda.synchronize()
    x32 = xg.float().cpu().numpy()
    del xg
    w = synth.Workload(name="c5_gpu_L%d_S%d" % (layer, site), x=x32, dtype="bf16", k=k, seed=seed)
    t0 = time.time()
    uo, vo = orc.decompose(x32.astype(np.float64), k, seed=seed)
    print("oracle decompose %.1fs" % (time.time() - t0), flush=True)
    # the factorisation is the oracle's full one; the m x n products are compared on every 16th
    # block of 64 rows (4160 rows, each computed exactly), U on all of its rows
    res = check_compress_parity(w, u, v, xhat, oracle_factors=(uo, vo), strict_ortho=True,
                                rows=sample_row_blocks(m, 16))
    print("c5 stream", layer, site, res, "status", int(status.item()))
    assert int(status.item()) == 0


def test_c4_rsvd_comparator():
    # config 4: same rank, oversampling 8, one power iteration, Gaussian test matrix from the seed
    import paper_2509_23472_amd as L
    w = synth.c4_mlp()
    p, q = w.extras["oversample"], w.extras["power_iters"]
    x = to_device(w.x, w.dtype)
    status = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    u, v = L.loract_rsvd(x, w.k, oversample=p, power_iters=q, seed=w.seed, status=status)
    torch.cuda.synchronize()
    t0 = time.time()
    omega_t = synth.round_to_bf16(orc.gaussian_omega_t(w.k + p, w.n, w.seed).astype(np.float32))
    uo, vo = orc.rsvd(w.x.astype(np.float64), w.k, oversample=p, power_iters=q,
                      omega_t=omega_t.astype(np.float64))
    print("oracle rsvd %.1fs" % (time.time() - t0), flush=True)
    res = check_compress_parity(w, u, v, oracle_factors=(uo, vo), strict_ortho=True)
    print("c4 rsvd", res, "status", int(status.item()))
    assert int(status.item()) == 0
    # both methods at equal rank on the same input: comparable approximation quality (Section 3.2)
    ul, vl = L.loract_compress(x, w.k, seed=w.seed)
    torch.cuda.synchronize()
    e_loract = orc.rel_fro(to_host(ul) @ to_host(vl), w.x.astype(np.float64))
    print("quality: loract %.4e  rsvd %.4e" % (e_loract, res["quality_gpu"]))
    # Section 3.2 claims comparable quality at equal rank; with oversampling and a power iteration
    # on its side the comparator may be better, but not by a different order of magnitude
    assert e_loract <= 3.0 * res["quality_gpu"]


def test_coherent_workload_sampling_versus_gaussian():
    # Second workload (outlier tokens with directions of their own, coherence at its maximum):
    # parity of both methods with the oracle, and the measured gap between row sampling and a
    # Gaussian test matrix at equal rank.  Theorem 4.3 ties the sampling error to the coherence but
    # the paper prints no number, so the gap is reported, not asserted; what is asserted is that
    # GPU and oracle agree on each method's loss and that more sampled rows (l = 2k) do not hurt.
    import paper_2509_23472_amd as L
    w = synth.coherent_activations(m=4096, n=1024, k=64, seed=6)
    x64 = w.x.astype(np.float64)
    x = to_device(w.x, w.dtype)
    status = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    u, v = L.loract_compress(x, w.k, seed=w.seed, status=status)
    ur, vr = L.loract_rsvd(x, w.k, oversample=0, power_iters=0, seed=w.seed)
    torch.cuda.synchronize()
    res = check_compress_parity(w, u, v)
    omega_t = synth.round_to_bf16(orc.gaussian_omega_t(w.k, w.n, w.seed).astype(np.float32))
    uo, vo = orc.rsvd(x64, w.k, omega_t=omega_t.astype(np.float64))
    res_r = check_compress_parity(w, ur, vr, oracle_factors=(uo, vo))
    print("coherent: sampling %.4e (oracle %.4e)  gaussian %.4e (oracle %.4e)  status %d" % (
        res["quality_gpu"], res["quality_oracle"], res_r["quality_gpu"], res_r["quality_oracle"],
        int(status.item())))
    # both sides agree on how much each method loses
    assert abs(res["quality_gpu"] - res["quality_oracle"]) <= 5e-3 * max(1.0, res["quality_oracle"])
    assert abs(res_r["quality_gpu"] - res_r["quality_oracle"]) <= 5e-3 * max(1.0, res_r["quality_oracle"])
    # more sampled rows (Theorem 4.3's l) close part of the gap
    u2, v2 = L.loract_compress(x, w.k, seed=w.seed, l=2 * w.k)
    torch.cuda.synchronize()
    e2 = orc.rel_fro(to_host(u2) @ to_host(v2), x64)
    print("coherent: sampling with l = 2k: %.4e" % e2)
    assert e2 <= res["quality_gpu"] * 1.02
