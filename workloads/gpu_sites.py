"""Long-context stream sites (config 5) generated on the GPU: harness code shared by bench.py and
the parity tests.  It holds none of the method's arithmetic -- only the seeded synthetic input.

A site is X = c (G1 diag(s)) G2^T + 1e-3 N with Gaussian G1 (m x p), G2 (n x p) scaled to
near-orthonormal columns, p = 1024 spectrum terms s_i = i^-1.5, c = sqrt(m n) / ||s||_2, N i.i.d.
standard normal, rounded to bf16; the per-site seed is 50000 + 7 layer + site.  Sites 0..5 of a
layer are 4096 wide (q/k/v/o and gate/up inputs), site 6 is the 11008-wide down-projection input.
Generating with torch's device generator keeps the 224-site stream off the host; a test that wants
the oracle's answer downloads the generated bits, so both sides still see identical inputs.
"""
from __future__ import annotations

import numpy as np

C5_ROWS = 16 * 4096
C5_RANK = 256
C5_TERMS = 1024
C5_WIDTHS = (4096, 4096, 4096, 4096, 4096, 4096, 11008)


def c5_site_seed(layer: int, site: int) -> int:
    return 50_000 + 7 * layer + site


def c5_site_on_gpu(torch, layer: int, site: int, out=None, m: int = C5_ROWS):
    """Fill `out` (a bf16 m x n view on the current device, allocated if None) with the site's
    activation matrix; the work is enqueued on torch's current stream."""
    n = C5_WIDTHS[site]
    p = C5_TERMS
    if out is None:
        out = torch.empty((m, n), dtype=torch.bfloat16, device="cuda")
    assert tuple(out.shape) == (m, n) and out.dtype == torch.bfloat16
    g = torch.Generator(device="cuda")
    g.manual_seed(c5_site_seed(layer, site))
    s = np.arange(1, p + 1, dtype=np.float64) ** -1.5
    c = float(np.sqrt(float(m) * n) / np.linalg.norm(s))
    svals = torch.arange(1, p + 1, device="cuda", dtype=torch.float32) ** -1.5
    g1 = torch.randn((m, p), generator=g, device="cuda", dtype=torch.float32) * (c / np.sqrt(m))
    g2 = torch.randn((n, p), generator=g, device="cuda", dtype=torch.float32) / np.sqrt(n)
    sig = ((g1 * svals).to(torch.bfloat16) @ g2.to(torch.bfloat16).t()).float()
    sig.add_(torch.randn((m, n), generator=g, device="cuda", dtype=torch.float32), alpha=1e-3)
    out.copy_(sig)
    return out
