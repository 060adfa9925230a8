"""Pins of the oracle's RoPE / YaRN functions (the checker of the fused RoPE + pooling producer)
and of its bf16 rounding, against what the paper and the mathematics fix."""
import math
import os

import numpy as np
import pytest

from oracle import prism_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_printed_values.txt")


def _golden():
    out = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            out[k.strip()] = float(v)
    return out


def test_frequencies_are_the_geometric_ladder():
    th = orc.rope_frequencies(128, 1.0e6)
    assert th.shape == (64,) and th[0] == 1.0
    assert np.allclose(th[1:] / th[:-1], 1.0e6 ** (-2.0 / 128), rtol=1e-13)   # constant ratio
    assert abs(th[32] - 1.0e-3) < 1e-15                                          # b^(-1/2)


def test_yarn_zone_boundaries_printed_in_the_appendix():
    g = _golden()
    base, d, L, s = 1.0e6, 128, 32768, 4.0
    th = orc.rope_frequencies(d, base)
    ty = orc.rope_frequencies(d, base, yarn=(L, s, 1.0, 32.0))
    two_j = 2 * np.arange(d // 2)
    unchanged = two_j[np.isclose(ty, th, rtol=0, atol=0)]
    full = two_j[np.isclose(ty, th / s, rtol=1e-15, atol=0)]
    # unchanged up to 2j ~ 47, fully scaled from 2j ~ 79 (even feature indices bracket the printed values)
    assert abs(unchanged.max() - g["yarn_unchanged_until_2j"]) <= 1.5
    assert abs(full.min() - g["yarn_full_scaling_from_2j"]) <= 1.5
    between = (two_j > unchanged.max()) & (two_j < full.min())
    assert (ty[between] < th[between]).all() and (ty[between] > th[between] / s).all()
    assert (np.diff(ty) < 0).all()                                   # still a decreasing ladder
    # r_j at the end of the dead zone (2j = 30) is about 2.0e2
    r30 = L * th[15] / (2 * math.pi)
    assert abs(r30 - g["yarn_r_at_dead_zone_end"]) / g["yarn_r_at_dead_zone_end"] < 0.05
    # the boundaries themselves: r = beta at theta = 2 pi beta / L, r = alpha at 2 pi alpha / L
    for r_edge, key in ((32.0, "yarn_unchanged_until_2j"), (1.0, "yarn_full_scaling_from_2j")):
        two_j_edge = -d * math.log(2 * math.pi * r_edge / L) / math.log(base)
        assert abs(two_j_edge - g[key]) < 0.5


def test_rope_is_a_rotation_with_the_right_sense_and_pairing():
    rng = np.random.default_rng(0)
    d, L = 16, 9
    X = rng.standard_normal((3, L, d))
    # quarter turn per position on every pair: (x, y) -> (-y, x) at position 1
    th = np.full(d // 2, math.pi / 2)
    R = orc.apply_rope(X, th)
    assert np.allclose(R[:, 0], X[:, 0], atol=1e-15)                           # position 0: identity
    assert np.allclose(R[:, 1, 0::2], -X[:, 1, 1::2], atol=1e-14)
    assert np.allclose(R[:, 1, 1::2], X[:, 1, 0::2], atol=1e-14)
    assert np.allclose(R[:, 2], -X[:, 2], atol=1e-14)                          # half turn at position 2
    # pairs are (2j, 2j+1): rotating only pair 3 leaves every other dim untouched
    th = np.zeros(d // 2); th[3] = 0.3
    R = orc.apply_rope(X, th)
    keep = np.ones(d, bool); keep[6:8] = False
    assert np.array_equal(R[..., keep], X[..., keep]) and not np.allclose(R[:, 1:, 6:8], X[:, 1:, 6:8])


def test_rope_preserves_norms_composes_and_depends_on_relative_position():
    rng = np.random.default_rng(1)
    d, L = 32, 40
    th = orc.rope_frequencies(d, 1.0e4)
    q, k = rng.standard_normal((L, d)), rng.standard_normal((L, d))
    Rq, Rk = orc.apply_rope(q, th), orc.apply_rope(k, th)
    assert np.allclose(np.linalg.norm(Rq.reshape(L, d // 2, 2), axis=-1),
                       np.linalg.norm(q.reshape(L, d // 2, 2), axis=-1), rtol=1e-13)
    # position offset = composition of rotations
    assert np.allclose(orc.apply_rope(q, th, position_offset=7)[:L - 7], orc.apply_rope(
        np.concatenate([np.zeros((7, d)), q])[None], th)[0][7:L], atol=1e-13)
    # <R_m a, R_n b> = <R_(m-n) a, b>
    a, b = q[0], k[0]
    A = orc.apply_rope(np.tile(a, (L, 1)), th)
    Bm = orc.apply_rope(np.tile(b, (L, 1)), th)
    for m, n in ((5, 2), (17, 17), (30, 11)):
        assert abs(A[m] @ Bm[n] - A[m - n] @ b) < 1e-12


@pytest.mark.parametrize("base,B", [(1.0e6, 128), (5.0e5, 64)])
def test_pooled_rope_of_constant_content_follows_the_dirichlet_kernel(base, B):
    """Eq. "attenuation": constant content c rotated by RoPE and mean-pooled over a block keeps the
    fraction |sin(B theta / 2) / (B sin(theta / 2))| of its magnitude."""
    d = 128
    th = orc.rope_frequencies(d, base)
    X = orc.apply_rope(np.ones((3 * B, d)), th)
    pooled = orc.pool(X[None], B)[0]                                         # [3, d]
    mag = np.linalg.norm(pooled.reshape(3, d // 2, 2), axis=-1) / math.sqrt(2.0)
    closed = np.abs(np.sin(B * th / 2) / np.sin(th / 2)) / B
    assert np.allclose(mag, closed[None, :], atol=1e-12)


def test_yarn_scaling_reduces_attenuation_only_beyond_the_unchanged_range():
    """The appendix' conclusion: dims up to 2j ~ 47 pool exactly as without YaRN; the scaled dims are
    attenuated less (their pooled magnitude grows), never more."""
    d, B, base = 128, 128, 1.0e6
    lam = lambda th: np.abs(np.sin(B * th / 2) / np.sin(th / 2)) / B
    th, ty = orc.rope_frequencies(d, base), orc.rope_frequencies(d, base, yarn=(32768, 4.0, 1.0, 32.0))
    l0, l1 = lam(th), lam(ty)
    assert np.array_equal(l0[:24], l1[:24])
    assert (l1[24:] >= l0[24:] - 1e-15).all() and (l1[30:] > l0[30:]).all()


def test_bf16_rounding_is_nearest_even():
    one = 1.0
    ulp = 2.0 ** -7
    x = np.array([one, one + ulp / 2, one + ulp, one + 1.5 * ulp, one + 0.4999 * ulp, one + 0.5001 * ulp,
                  -(one + 1.5 * ulp), 0.0, 3.0e38, 1e-40])
    bits = orc.f64_to_bf16_bits(x)
    back = orc.bf16_to_f64(bits)
    assert back[0] == one and back[1] == one            # tie -> even mantissa (1.0)
    assert back[2] == one + ulp and back[3] == one + 2 * ulp   # tie -> even (1 + 2 ulp)
    assert back[4] == one and back[5] == one + ulp and back[6] == -(one + 2 * ulp) and back[7] == 0.0
    rng = np.random.default_rng(2)
    y = rng.standard_normal(100000) * np.exp(3 * rng.standard_normal(100000))
    yb = orc.bf16_to_f64(orc.f64_to_bf16_bits(y))
    assert (np.abs(yb - y) <= np.abs(y) * 2.0 ** -8 * (1 + 1e-12)).all()          # within half an ulp
    assert np.array_equal(orc.f64_to_bf16_bits(yb), orc.f64_to_bf16_bits(yb))     # idempotent
