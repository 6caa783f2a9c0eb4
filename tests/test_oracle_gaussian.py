"""Pins for the uniform -> normal map of the oracle's noise field."""
import math

import numpy as np
from scipy import stats

from oracle import flashdp_oracle as O


def test_uniform24_range_and_grid():
    r = np.array([0, 255, 256, 0xFFFFFFFF, 0x80000000], dtype=np.uint32)
    u = O.uniform24(r)
    assert u[0] == 2.0 ** -25 and u[1] == 2.0 ** -25      # low 8 bits are dropped
    assert u[2] == 1.5 * 2.0 ** -24
    assert u[3] == 1.0 - 2.0 ** -25                        # never reaches 1
    assert u[4] == 0.5 + 2.0 ** -25
    assert np.all((u > 0) & (u < 1))


def test_box_muller_closed_form_points():
    # r0 = r1 = 0: u = 2^-25 -> rho = sqrt(50 ln 2); angle 2 pi 2^-25
    z = O.gaussians_from_words(np.array([0, 0, 0, 0], np.uint32))
    rho = math.sqrt(50.0 * math.log(2.0))
    ang = 2.0 * math.pi * 2.0 ** -25
    assert abs(z[0] - rho * math.cos(ang)) < 1e-14
    assert abs(z[1] - rho * math.sin(ang)) < 1e-20 + 1e-14 * abs(z[1])
    assert z[1] > 0 and z[1] < 2e-6                      # sine on slot 1, cosine on slot 0
    assert z[2] == z[0] and z[3] == z[1]                  # second pair uses (r2, r3) the same way
    # quarter turn: u1 = 1/4 + 2^-25 -> cos ~ 0-, sin ~ 1 ; radius from r0 = 2^31: u0 = 1/2 + 2^-25
    r = np.array([1 << 31, 1 << 30, 0, 1 << 31], np.uint32)
    z = O.gaussians_from_words(r)
    rho = math.sqrt(-2.0 * math.log(0.5 + 2.0 ** -25))
    assert abs(z[1] - rho) < 1e-12 and abs(z[0]) < 1e-6 and z[0] < 0
    # half turn on the second pair with the largest radius: z2 ~ -rho_max, z3 ~ 0-
    assert abs(z[2] + math.sqrt(50.0 * math.log(2.0))) < 1e-12 and z[3] < 0 and abs(z[3]) < 1e-5
    # radius uses the FIRST word of each pair, angle the second
    a = O.gaussians_from_words(np.array([5 << 8, 9 << 8, 0, 0], np.uint32))
    b = O.gaussians_from_words(np.array([9 << 8, 5 << 8, 0, 0], np.uint32))
    assert abs(math.hypot(a[0], a[1]) - math.sqrt(-2 * math.log(5.5 / 2 ** 24))) < 1e-12
    assert abs(math.hypot(b[0], b[1]) - math.sqrt(-2 * math.log(9.5 / 2 ** 24))) < 1e-12


def test_field_is_standard_normal():
    n = 1_000_000
    z = O.noise_field(20250701, 3, n)
    assert abs(z.mean()) < 4.0 / math.sqrt(n)
    assert abs(z.var() - 1.0) < 4.0 * math.sqrt(2.0 / n)
    assert abs(stats.skew(z)) < 0.01
    assert abs(stats.kurtosis(z)) < 0.02
    assert np.max(np.abs(z)) <= math.sqrt(50.0 * math.log(2.0)) + 1e-12
    ks = stats.kstest(z, "norm")
    assert ks.pvalue > 1e-3, ks
    # each of the four slots alone is standard normal, and slots are uncorrelated
    z4 = z.reshape(-1, 4)
    for j in range(4):
        assert stats.kstest(z4[:, j], "norm").pvalue > 1e-3
    corr = np.corrcoef(z4.T)
    assert np.max(np.abs(corr - np.eye(4))) < 0.01
    # neighbouring groups are uncorrelated too
    assert abs(np.corrcoef(z4[:-1, 0], z4[1:, 0])[0, 1]) < 0.01
