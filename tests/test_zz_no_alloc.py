"""loract_lora_grad_static: the entry point that allocates nothing (its scratch is a buffer built
into the library's device image).  Called through the C ABI binding and compared, bit for bit,
with loract_lora_grad on the same factors: two calls in a row, the second on a smaller input, so
that whatever the first call left in the shared buffer is there when the second one runs.
"""
import numpy as np
import pytest
import torch

from workloads import synth

from gpu_util import to_device

pytestmark = pytest.mark.gpu


def _case(L, m, n, k, n_out, r, seed):
    s = 0.9 ** np.arange(min(m, n))
    x = synth.round_to_bf16(synth.spectrum_matrix(m, n, s, 1e-3, seed).astype(np.float32))
    rng = np.random.default_rng(seed)
    dy = synth.round_to_bf16(rng.standard_normal((m, n_out)).astype(np.float32))
    b = synth.round_to_bf16((rng.standard_normal((r, n_out)) / np.sqrt(r)).astype(np.float32))
    u, v = L.loract_compress(to_device(x, "bf16"), k, seed=seed)
    return u, v, to_device(dy, "bf16"), to_device(b, "bf16")


def test_static_scratch_entry_matches_workspace_entry_on_two_calls_in_a_row():
    import paper_2509_23472_amd as L
    assert L.loract_static_scratch_bytes() == 16 << 20
    big = _case(L, 2048, 1024, 64, 1024, 16, 1)        # matrix-core path, 1.1 MiB of scratch
    small = _case(L, 300, 136, 20, 75, 5, 2)           # ragged shapes: the generic kernels
    mid = _case(L, 777, 256, 32, 320, 16, 3)
    outs = {}
    for name, (u, v, dy, b) in (("big", big), ("small", small), ("mid", mid)):
        outs[name] = (L.loract_lora_grad(u, v, dy, b, scale=0.5).clone(),
                      torch.full((v.shape[1], b.shape[0]), float("nan"), dtype=torch.float32, device="cuda"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for name, (u, v, dy, b) in (("big", big), ("small", small), ("mid", mid), ("big", big)):
        print("static call", name, tuple(u.shape), tuple(dy.shape), flush=True)
        outs[name][1].fill_(float("nan"))
        L.loract_lora_grad_static(u, v, dy, b, outs[name][1], scale=0.5)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before          # nothing allocated through torch either
        assert torch.equal(outs[name][1], outs[name][0]), name   # same kernels, same plan: bit-identical
