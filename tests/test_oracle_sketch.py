"""Pins for the oracle's sketch generator (Algorithm 1, sampling step: normal
entries of variance 1/r; Section 3.2).  CPU only."""

import math
import os

import numpy as np
import pytest
from scipy import stats

from oracle import curdkv_oracle as orc

M64 = (1 << 64) - 1


def test_splitmix64_published_vector(golden_dir):
    want = [int(x) for x in open(os.path.join(golden_dir, "splitmix64_seed1234567.txt"))
            if x.strip() and not x.startswith("#")]
    got = orc.splitmix64_outputs(1234567, 1, len(want))
    assert [int(x) for x in got] == want


def test_splitmix64_is_random_access():
    a = orc.splitmix64_outputs(99, 1, 1000)
    b = orc.splitmix64_outputs(99, 501, 20)
    assert np.array_equal(a[500:520], b)


def _scalar_mix(z):
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def _scalar_element(seed, layer, head, H, d, r, i, j):
    """One element of G by scalar Python arithmetic, from the generator's
    definition: counter -> two words -> Box-Muller -> scale (before rounding)."""
    c = ((layer * H + head) * d + i) * r + j
    g = 0x9E3779B97F4A7C15
    w1 = _scalar_mix((seed + (2 * c + 1) * g) & M64)
    w2 = _scalar_mix((seed + (2 * c + 2) * g) & M64)
    u1 = ((w1 >> 11) + 1) * 2.0 ** -53
    u2 = (w2 >> 11) * 2.0 ** -53
    return math.sqrt(-2.0 * math.log(u1)) * math.cos(2.0 * math.pi * u2) / math.sqrt(r)


@pytest.mark.parametrize("dtype,tol", [("fp32", 2.0 ** -23), ("bf16", 2.0 ** -8)])
def test_sketch_counter_addressing(dtype, tol):
    seed, H, d, r = 0xC0DE0003, 8, 128, 64
    for (l, h) in [(0, 0), (0, 7), (3, 2), (31, 7)]:
        G = orc.sketch(seed, l, h, H, d, r, dtype)
        assert G.shape == (d, r)
        for (i, j) in [(0, 0), (0, 1), (1, 0), (127, 63), (64, 17)]:
            want = _scalar_element(seed, l, h, H, d, r, i, j)
            assert abs(G[i, j] - want) <= tol * abs(want) + 1e-300, (l, h, i, j)


def test_sketch_distinct_per_group_and_shared_by_nothing_else():
    a = orc.sketch(1, 0, 0, 8, 128, 64, "bf16")
    b = orc.sketch(1, 0, 1, 8, 128, 64, "bf16")
    c = orc.sketch(1, 1, 0, 8, 128, 64, "bf16")
    d = orc.sketch(2, 0, 0, 8, 128, 64, "bf16")
    assert not np.array_equal(a, b) and not np.array_equal(a, c) and not np.array_equal(a, d)
    assert np.array_equal(a, orc.sketch(1, 0, 0, 8, 128, 64, "bf16"))
    # consecutive groups use consecutive, non-overlapping counter ranges
    assert abs(np.corrcoef(a.ravel(), b.ravel())[0, 1]) < 0.05


@pytest.mark.parametrize("r", [20, 32, 64, 128])
def test_sketch_moments_and_normality(r):
    d, H = 128, 8
    G = np.stack([orc.sketch(0xABCDEF, l, h, H, d, r, "fp32")
                  for l in range(4) for h in range(H)])
    x = G.ravel() * math.sqrt(r)          # should be N(0, 1)
    N = x.size
    assert abs(x.mean()) < 5.0 / math.sqrt(N)
    assert abs(x.var() - 1.0) < 5.0 * math.sqrt(2.0 / N)
    assert abs(stats.skew(x)) < 0.05 and abs(stats.kurtosis(x)) < 0.1
    assert stats.kstest(x[:200000], "norm").pvalue > 1e-3
    # E[G G^T] = I_d  (variance 1/r per entry, r entries per row product)
    GGt = np.mean(G @ np.transpose(G, (0, 2, 1)), axis=0)
    assert np.allclose(np.diag(GGt), 1.0, atol=6.0 * math.sqrt(2.0 / (r * 32)))
    off = GGt - np.diag(np.diag(GGt))
    assert np.abs(off).max() < 6.0 / math.sqrt(r * 32)


def test_storage_rounding():
    # bf16 RNE: ties go to the even mantissa
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20,
                  -1.0 - 2.0 ** -8, 3.0e-39], dtype=np.float32)
    bits = orc.f32_to_bf16_bits(x)
    back = orc.bf16_bits_to_f64(bits)
    assert back[0] == 1.0
    assert back[1] == 1.0                      # tie -> even (mantissa 0)
    assert back[2] == 1.0 + 2.0 ** -6          # tie -> even (mantissa 2)
    assert back[3] == 1.0 + 2.0 ** -7          # above the tie -> up
    assert back[4] == -1.0
    # every bf16 value survives a round trip exactly
    allbits = np.arange(0, 0x7F80, dtype=np.uint16)
    v = orc.bf16_bits_to_f64(allbits).astype(np.float32)
    assert np.array_equal(orc.f32_to_bf16_bits(v), allbits)
    # sketch values are representable in the storage type
    G = orc.sketch(5, 0, 0, 1, 128, 32, "bf16").astype(np.float32)
    assert np.all((G.view(np.uint32) & 0xFFFF) == 0)
    G32 = orc.sketch(5, 0, 0, 1, 128, 32, "fp32")
    assert np.array_equal(G32, G32.astype(np.float32).astype(np.float64))
    # rounding moves a value by at most half an ulp of the storage type
    Gb = orc.sketch(5, 0, 0, 1, 128, 32, "bf16")
    assert np.max(np.abs(Gb - G32) / np.abs(G32)) <= 2.0 ** -8
