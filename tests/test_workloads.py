"""Checks of the seeded input generators (no arithmetic of the method lives there; these tests pin
the properties the workloads are supposed to have)."""
import numpy as np

from workloads import synth


def test_bf16_round_trip_is_exact_and_nearest_even():
    x = np.array([1.0, 1.00390625, 1.005859375, -3.140625, 0.0, 65280.0], dtype=np.float32)
    bits = synth.f32_to_bf16_bits(x)
    back = synth.bf16_bits_to_f32(bits)
    assert np.array_equal(synth.f32_to_bf16_bits(back), bits)
    # 1 + 2^-8 lies halfway between 1 and 1 + 2^-7: ties go to the even mantissa (1.0)
    assert back[1] == 1.0
    assert back[2] == np.float32(1.0078125)


def test_rank_k_floor_matches_the_singular_values_of_the_generated_matrix():
    for w, k in ((synth.c2_vit(m=1000, n=300, k=32), 32), (synth.c3_llama(m=1024, n=512, k=64), 64)):
        s = np.linalg.svd(w.x.astype(np.float64), compute_uv=False)
        optimum = np.sqrt(np.sum(s[k:] ** 2) / np.sum(s ** 2))
        assert abs(w.extras["rank_k_floor"] - optimum) <= 0.03 * optimum


def test_coherent_workload_has_leading_directions_on_single_rows():
    w = synth.coherent_activations(m=512, n=256, k=16, seed=6, outlier_rows=4)
    x = w.x.astype(np.float64)
    u, s, _ = np.linalg.svd(x, full_matrices=False)
    rows = w.extras["outlier_rows"]
    # the 4 leading left singular vectors live on the 4 outlier rows, and dominate the spectrum
    mass = np.sum(u[rows, :4] ** 2)
    assert mass >= 0.99 * 4
    assert s[3] >= 3 * s[4]
    # coherence of the leading k-dimensional subspace, (m/k) max_i ||U_k[i,:]||^2, is near its maximum m/k
    mu = (512 / 16) * np.max(np.sum(u[:, :16] ** 2, axis=1))
    assert mu >= 0.9 * 512 / 16


def test_workloads_are_reproducible_from_their_seed():
    a = synth.c5_long_context_site(1, 2, m=256, n=128, k=8)
    b = synth.c5_long_context_site(1, 2, m=256, n=128, k=8)
    c = synth.c5_long_context_site(1, 3, m=256, n=128, k=8)
    assert np.array_equal(a.x, b.x) and not np.array_equal(a.x, c.x)
