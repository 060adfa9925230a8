"""Pins for the selection half of the CPU oracle (no GPU).

Each test checks oracle/prism_oracle.py against something other than itself:
closed forms and values the paper prints (tests/golden/paper_printed_values.txt),
scalar brute force on tiny inputs, library routines for special cases, and
invariants of top-p.
"""
import itertools
import math
import os

import numpy as np
import pytest
import torch

from oracle import prism_oracle as orc
from paper_2602_08426_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_printed_values.txt")


def _golden():
    vals = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if "=" in line:
                k, v = line.split("=")
                vals[k.strip()] = float(v)
    return vals


# --------------------------------------------------------------------------- #
# pooling under RoPE: Dirichlet-kernel closed form (Eq. "attenuation")
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("base", [1.0e4, 5.0e5, 1.0e6])
@pytest.mark.parametrize("B", [64, 128])
@pytest.mark.parametrize("n0_blocks", [0, 3, 17])
def test_pool_matches_dirichlet_closed_form(base, B, n0_blocks):
    d = 128
    rng = np.random.default_rng(7)
    content = rng.standard_normal(d)
    L = (n0_blocks + 1) * B
    X = wl.constant_content_rope(content, np.arange(L), base)[None]       # [1, L, d]
    pooled = orc.pool(X, B)[0, n0_blocks]                                  # block starting at n0
    mag = np.hypot(pooled[0::2], pooled[1::2])
    cmag = np.hypot(content[0::2], content[1::2])
    theta = base ** (-2.0 * np.arange(d // 2) / d)
    closed = np.abs(np.sin(B * theta / 2) / np.sin(theta / 2)) / B
    np.testing.assert_allclose(mag / cmag, closed, rtol=0, atol=1e-12)


def test_pool_phase_is_block_start_times_geometric_sum():
    """Geometric-summation form of Sec. 3.2: pooled pair = c e^{i n0 th} (1/B) sum_k e^{i k th}."""
    d, B, base, n0 = 16, 8, 100.0, 24
    content = np.arange(1, d + 1, dtype=np.float64)
    X = wl.constant_content_rope(content, np.arange(n0 + B), base)[None]
    pooled = orc.pool(X, B)[0, n0 // B]
    for j in range(d // 2):
        th = base ** (-2.0 * j / d)
        c = complex(content[2 * j], content[2 * j + 1])
        expect = c * np.exp(1j * n0 * th) * sum(np.exp(1j * k * th) for k in range(B)) / B
        assert abs(complex(pooled[2 * j], pooled[2 * j + 1]) - expect) < 1e-12


def test_printed_cutoffs_and_theta():
    g = _golden()
    # The printed feature index 2j solves B * theta = 2*pi (Eq. "dim-cal"): a pair rotating at
    # theta = base^(-2j/d) for that (fractional) index must pool to (almost) nothing, and
    # pairs two dims to either side must not.
    for base, B, d, key in [(1.0e6, 128, 128, "cutoff_2j_base1e6_B128_d128"),
                            (256.0, 128, 16, "cutoff_2j_base256_B128_da16"),
                            (256.0, 128, 56, "cutoff_2j_base256_B128_da56")]:
        def pooled_mag(two_j):
            th = base ** (-two_j / d)
            n = np.arange(B)
            X = np.stack([np.cos(n * th), np.sin(n * th)], axis=1)[None]      # [1, B, 2]
            pb = orc.pool(X, B)[0, 0]
            return float(np.hypot(pb[0], pb[1]))
        printed = g[key]
        assert pooled_mag(printed) < 0.03, (key, pooled_mag(printed))
        assert pooled_mag(printed + 0.25 * d / 16) > pooled_mag(printed)
        assert pooled_mag(printed - 0.25 * d / 16) > pooled_mag(printed)
    theta10 = wl.rope_frequencies(128, 1.0e6)[10]
    assert abs(theta10 - g["theta_10_base1e6_d128"]) < 0.01
    x = theta10 / 2
    assert abs(math.sin(x) - x) / math.sin(x) < g["sinc_rel_err_bound_at_theta_10"]


def test_zones_dead_and_semantic():
    g = _golden()
    d, B, base = 128, 128, 1.0e6
    X = wl.constant_content_rope(np.ones(d), np.arange(4 * B), base)[None]
    pooled = orc.pool(X, B)[0]                       # [4, d]
    mag = np.hypot(pooled[:, 0::2], pooled[:, 1::2]) / math.sqrt(2.0)
    dead = int(g["dead_zone_end_2j"]) // 2
    sem = int(g["semantic_zone_start_2j"]) // 2
    assert mag[:, :dead - 1].max() < 0.25            # collapsed
    assert mag[:, sem:].min() > 0.9                  # preserved


def test_iid_content_pooled_rms_is_one_over_sqrt_B():
    g = _golden()
    rng = np.random.default_rng(3)
    B, d, N = 128, 128, 64
    X = rng.standard_normal((1, N * B, d))
    r = orc.rms(orc.pool(X, B))[0]
    assert abs(r - g["residual_rms_factor_B128"]) < 0.002
    assert abs(r - 1 / math.sqrt(B)) < 3 * (1 / math.sqrt(B)) / math.sqrt(2 * N * d)


def test_pool_ragged_tail_divides_by_actual_count():
    X = np.arange(2 * 7 * 3, dtype=np.float64).reshape(2, 7, 3)
    pb = orc.pool(X, 3)
    assert pb.shape == (2, 3, 3)
    np.testing.assert_allclose(pb[:, 2], X[:, 6], atol=0)
    np.testing.assert_allclose(pb[:, 0], (X[:, 0] + X[:, 1] + X[:, 2]) / 3, atol=1e-15)


# --------------------------------------------------------------------------- #
# scalar brute force of the whole selection on tiny inputs
# --------------------------------------------------------------------------- #
def _scalar_prism(Q, K, d_h, d_l, B, p, calibrate=True, causal=True, dims=None):
    """Index-by-index restatement of Sec. 3.4 with Python scalars (tiny sizes only).
    `dims` optionally gives the feature dims of each band explicitly."""
    h, L, d = len(Q), len(Q[0]), len(Q[0][0])
    h_kv = len(K)
    g = h // h_kv
    N = L // B

    def pooled(X):
        return [[[sum(X[a][u * B + t][c] for t in range(B)) / B for c in range(d)]
                 for u in range(N)] for a in range(len(X))]

    Qb, Kb = pooled(Q), pooled(K)

    def band(z):
        if dims is not None:
            return list(dims[z])
        return list(range(0, d_h)) if z == "high" else list(range(d - d_l, d))

    def rms_of(Xb_head, dims):
        tot = 0.0
        for u in range(N):
            for c in dims:
                tot += Xb_head[u][c] ** 2
        return math.sqrt(tot / (N * len(dims)))

    masks = {}
    logits = {}
    for z in ("high", "low"):
        zdims = band(z)
        dz = len(zdims)
        M = [[[False] * N for _ in range(N)] for _ in range(h)]
        Lg = [[[-math.inf] * N for _ in range(N)] for _ in range(h)]
        for hq in range(h):
            kv = hq // g
            if calibrate:
                tau = math.sqrt(dz / d) * (rms_of(Qb[hq], zdims) / rms_of(Qb[hq], range(d))) \
                    * (rms_of(Kb[kv], zdims) / rms_of(Kb[kv], range(d)))
            else:
                tau = 1.0
            for u in range(N):
                row = []
                nvis = u + 1 if causal else N
                for v in range(nvis):
                    dot = sum(Qb[hq][u][c] * Kb[kv][v][c] for c in zdims)
                    row.append(dot / (tau * math.sqrt(dz)))
                    Lg[hq][u][v] = row[-1]
                mx = max(row)
                ex = [math.exp(x - mx) for x in row]
                s = sum(ex)
                pr = [e / s for e in ex]
                order = sorted(range(nvis), key=lambda i: (-pr[i], i))
                before = 0.0
                for i in order:
                    if before < p:
                        M[hq][u][i] = True
                    before += pr[i]
        masks[z] = M
        logits[z] = Lg
    return masks, logits


@pytest.mark.parametrize("seed,h,h_kv,d,d_h,d_l,B,N,p", [
    (0, 1, 1, 8, 4, 6, 2, 5, 0.7),
    (1, 4, 2, 8, 2, 4, 3, 6, 0.9),
    (2, 2, 1, 12, 8, 8, 4, 7, 0.5),
    (3, 6, 2, 8, 8, 8, 2, 4, 0.95),
])
def test_selection_matches_scalar_brute_force(seed, h, h_kv, d, d_h, d_l, B, N, p):
    rng = np.random.default_rng(seed)
    L = B * N
    Q = rng.standard_normal((h, L, d)) * 3.0
    K = rng.standard_normal((h_kv, L, d)) * 3.0
    sel = orc.prism_select(Q, K, d_h, d_l, B, p)
    masks, logits = _scalar_prism(Q.tolist(), K.tolist(), d_h, d_l, B, p)
    for z in ("high", "low"):
        np.testing.assert_array_equal(sel.band_masks[z], np.array(masks[z]))
        lg = np.array(logits[z])
        fin = np.isfinite(lg)
        np.testing.assert_array_equal(np.isfinite(sel.logits[z]), fin)
        np.testing.assert_allclose(sel.logits[z][fin], lg[fin], rtol=1e-12, atol=1e-12)
    union = np.array(masks["high"]) | np.array(masks["low"])
    np.testing.assert_array_equal(sel.mask, union)


@pytest.mark.parametrize("seed,causal", [(10, True), (11, False), (12, False)])
def test_segment_bands_and_bidirectional_match_scalar_brute_force(seed, causal):
    """Bands given as lists of slices (axis-wise bands of App. "HunyuanVideo Spectral
    Configuration": first d_high^a / last d_low^a dims of each axis subspace) and the
    bidirectional variant, against the scalar restatement."""
    rng = np.random.default_rng(seed)
    h, h_kv, d, B, N, p = 4, 2, 16, 2, 6, 0.8
    # three axis subspaces [4, 6, 6]: high = first 2 / 3 / 3 dims, low = last 4 / 4 / 4
    bands = {"high": [(0, 2), (4, 3), (10, 3)], "low": [(0, 4), (6, 4), (12, 4)]}
    dims = {z: [c for s0, w in segs for c in range(s0, s0 + w)] for z, segs in bands.items()}
    Q = rng.standard_normal((h, B * N, d)) * 3.0
    K = rng.standard_normal((h_kv, B * N, d)) * 3.0
    sel = orc.prism_select(Q, K, 0, 0, B, p, causal=causal, bands=bands)
    masks, logits = _scalar_prism(Q.tolist(), K.tolist(), 0, 0, B, p, causal=causal, dims=dims)
    for z in ("high", "low"):
        np.testing.assert_array_equal(sel.band_masks[z], np.array(masks[z]))
        lg = np.array(logits[z])
        fin = np.isfinite(lg)
        np.testing.assert_array_equal(np.isfinite(sel.logits[z]), fin)
        np.testing.assert_allclose(sel.logits[z][fin], lg[fin], rtol=1e-12, atol=1e-12)
    if not causal:
        assert np.isfinite(sel.logits["high"]).all() and sel.mask[:, 0, :].sum() >= h


def test_single_slice_descriptor_is_the_default_and_dims_may_be_permuted():
    """One slice per band == the d_h / d_l form; permuting the feature dims of Q and K
    together with the band descriptors leaves every logit unchanged."""
    rng = np.random.default_rng(21)
    h, h_kv, d, B, N, p = 2, 1, 16, 4, 8, 0.9
    Q = rng.standard_normal((h, B * N, d)); K = rng.standard_normal((h_kv, B * N, d))
    a = orc.prism_select(Q, K, 8, 12, B, p)
    b = orc.prism_select(Q, K, 0, 0, B, p, bands={"high": [(0, 8)], "low": [(4, 12)]})
    np.testing.assert_array_equal(a.mask, b.mask)
    np.testing.assert_array_equal(a.logits["low"], b.logits["low"])
    # half-split storage: pair j lives in dims (j, j + d/2) instead of (2j, 2j+1)
    to_half = np.concatenate([np.arange(0, d, 2), np.arange(1, d, 2)])   # new dim i holds old dim to_half[i]
    Qp, Kp = Q[:, :, to_half], K[:, :, to_half]
    half = {"high": [(0, 4), (8, 4)], "low": [(2, 6), (10, 6)]}          # pairs 0..3 and pairs 2..7
    c = orc.prism_select(Qp, Kp, 0, 0, B, p, bands=half)
    for z in ("high", "low"):
        fin = np.isfinite(a.logits[z])
        np.testing.assert_allclose(c.logits[z][fin], a.logits[z][fin], rtol=1e-12, atol=1e-12)
    np.testing.assert_array_equal(c.mask, a.mask)
    with pytest.raises(ValueError):
        orc.band_dims(d, 0, 0, {"high": [(0, 8), (4, 8)], "low": []})     # overlapping slices
    with pytest.raises(ValueError):
        orc.band_dims(d, 0, 0, {"high": [(12, 8)], "low": []})            # runs past the head dim


def test_forced_blocks_are_added_after_the_union():
    rng = np.random.default_rng(22)
    h, h_kv, d, B, N, p = 2, 1, 8, 2, 9, 0.3
    Q = rng.standard_normal((h, B * N, d)) * 4; K = rng.standard_normal((h_kv, B * N, d)) * 4
    base = orc.prism_select(Q, K, 4, 4, B, p)
    forced = orc.prism_select(Q, K, 4, 4, B, p, force_diagonal=True, force_sink=True)
    eye = np.eye(N, dtype=bool)[None]
    sink = np.zeros((1, N, N), bool); sink[:, :, 0] = True
    np.testing.assert_array_equal(forced.mask, base.mask | eye | sink)
    assert not base.forced.any() and (forced.mask & ~base.mask).any()
    tol = orc.selection_tolerance(forced, p)
    assert (tol.must & (eye | sink)).sum() == (eye | sink).sum() * h      # forced blocks are never "don't care"
    assert not (tol.must & tol.must_not).any()


def test_band_slices_are_first_dh_and_last_dl():
    """Energy only in dims the high band cannot see -> high band flat (selects ~p of the
    causal row), low band sees it.  Catches a swapped / shifted slice."""
    h, d, B, N = 1, 16, 2, 8
    L = B * N
    rng = np.random.default_rng(0)
    Q = np.zeros((h, L, d)); K = np.zeros((h, L, d))
    Q[..., 12:] = 1.0 + 0.01 * rng.standard_normal((h, L, 4))
    K[..., 12:] = rng.standard_normal((h, L, 4)) * 5
    Q[..., :4] = 1e-9 * rng.standard_normal((h, L, 4))     # nearly no high-band energy
    K[..., :4] = 1e-9 * rng.standard_normal((h, L, 4))
    sel = orc.prism_select(Q, K, d_h=4, d_l=4, B=B, p=0.6, calibrate=False)
    # uncalibrated: high logits ~1e-18 -> uniform -> picks ceil(0.6*(u+1)) lowest indices
    for u in range(N):
        k = math.ceil(0.6 * (u + 1) - 1e-9)
        assert sel.band_masks["high"][0, u, :u + 1].sum() == k
        assert sel.band_masks["high"][0, u, :k].all()
    # low band logits equal the dims 12..15 dot products
    Qb = Q.reshape(h, N, B, d).mean(2); Kb = K.reshape(h, N, B, d).mean(2)
    ref = torch.from_numpy(Qb[0, :, 12:]) @ torch.from_numpy(Kb[0, :, 12:]).T / math.sqrt(4)
    tri = np.tril(np.ones((N, N), bool))
    np.testing.assert_allclose(sel.logits["low"][0][tri], ref.numpy()[tri], rtol=1e-13)


# --------------------------------------------------------------------------- #
# calibration special cases
# --------------------------------------------------------------------------- #
def test_full_width_bands_reduce_to_coarse_attention():
    """d_h = d_l = d  =>  tau = 1 and both bands equal softmax(Qbar Kbar^T / sqrt(d))."""
    rng = np.random.default_rng(11)
    h, h_kv, d, B, N = 4, 2, 32, 4, 9
    Q = rng.standard_normal((h, B * N, d)); K = rng.standard_normal((h_kv, B * N, d))
    sel = orc.prism_select(Q, K, d, d, B, 0.8)
    np.testing.assert_allclose(sel.tau["high"], 1.0, rtol=1e-14)
    np.testing.assert_allclose(sel.tau["low"], 1.0, rtol=1e-14)
    Qb = torch.from_numpy(Q).reshape(h, N, B, d).mean(2)
    Kb = torch.from_numpy(K).reshape(h_kv, N, B, d).mean(2).repeat_interleave(h // h_kv, 0)
    s = Qb @ Kb.transpose(1, 2) / math.sqrt(d)
    s = s.masked_fill(~torch.tril(torch.ones(N, N, dtype=torch.bool)), float("-inf"))
    P = torch.softmax(s, dim=-1).numpy()
    np.testing.assert_allclose(sel.probs["high"], P, atol=1e-14)
    np.testing.assert_allclose(sel.probs["low"], P, atol=1e-14)
    np.testing.assert_array_equal(sel.band_masks["high"], sel.band_masks["low"])


def test_scale_identity_and_homogeneity():
    rng = np.random.default_rng(5)
    h, h_kv, d, d_h, d_l, B, N = 4, 2, 32, 16, 24, 4, 8
    Q = rng.standard_normal((h, B * N, d)); K = rng.standard_normal((h_kv, B * N, d))
    s1 = orc.prism_select(Q, K, d_h, d_l, B, 0.9)
    # scale_z = (d_z / sqrt(d)) (rq_z rk_z) / (rq rk)
    kv = np.arange(h) // (h // h_kv)
    for z, dz in (("high", d_h), ("low", d_l)):
        alt = (dz / math.sqrt(d)) * s1.rms_q[z] * s1.rms_k[z][kv] / (s1.rms_q["full"] * s1.rms_k["full"][kv])
        np.testing.assert_allclose(s1.scale[z], alt, rtol=1e-13)
    # tau depends on energy ratios only: scaling Q by alpha leaves tau, scales logits by alpha
    s2 = orc.prism_select(3.0 * Q, K, d_h, d_l, B, 0.9)
    tri = np.tril(np.ones((N, N), bool))
    for z in ("high", "low"):
        np.testing.assert_allclose(s2.tau[z], s1.tau[z], rtol=1e-13)
        np.testing.assert_allclose(s2.logits[z][:, tri], 3.0 * s1.logits[z][:, tri], rtol=1e-12)


def test_rms_definition_against_frobenius_norm():
    rng = np.random.default_rng(2)
    X = rng.standard_normal((3, 10, 6))
    r = orc.rms(X)
    for a in range(3):
        assert abs(r[a] - np.linalg.norm(X[a]) / math.sqrt(10 * 6)) < 1e-14


def test_calibration_restores_band_logit_scale():
    """|L_z| / tau_z ~ |L_full| (approximate; Sec. 3.4).  Report-level check: within 2x."""
    w = wl.small_variant(wl.WORKLOADS["c2_llama_8k"], 4096, 4, 1)
    Qb, Kb, _ = wl.generate(w, n_threads=1)
    Q, K = orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb)
    sel = orc.prism_select(Q, K, 64, 96, 128, 0.95)
    N = w.n_blocks
    full = np.einsum("hud,vd->huv", sel.q_pooled, sel.k_pooled[0]) / math.sqrt(128)
    tri = np.tril(np.ones((N, N), bool))
    for z in ("high", "low"):
        for hq in range(4):
            a = np.sqrt(np.mean(sel.logits[z][hq][tri] ** 2))
            b = np.sqrt(np.mean(full[hq][tri] ** 2))
            assert 0.3 < a / b < 3.0, (z, hq, a, b)


# --------------------------------------------------------------------------- #
# top-p
# --------------------------------------------------------------------------- #
def test_top_p_brute_force_subsets():
    rng = np.random.default_rng(9)
    for trial in range(60):
        n = int(rng.integers(1, 11))
        pr = rng.dirichlet(np.ones(n) * rng.uniform(0.2, 2.0))
        p = float(rng.uniform(0.05, 0.999))
        got = orc.top_p(pr[None], p)[0]
        # brute force: smallest cardinality with mass >= p, and among those the largest mass
        best = None
        for k in range(1, n + 1):
            cands = [(sum(pr[list(c)]), c) for c in itertools.combinations(range(n), k)]
            m, c = max(cands)
            if m >= p or k == n:
                best = set(c)
                break
        assert set(np.nonzero(got)[0]) == best, (pr, p)


def test_top_p_invariants():
    rng = np.random.default_rng(4)
    P = rng.dirichlet(np.ones(40) * 0.3, size=200)
    for p in (0.1, 0.5, 0.93, 0.95, 0.999):
        M = orc.top_p(P, p)
        assert (M.sum(1) >= 1).all()
        mass = (P * M).sum(1)
        assert (mass >= p - 1e-12).all()
        smallest = np.where(M, P, np.inf).min(1)
        assert (mass - smallest < p).all()                 # minimality
        # selected are the largest ones
        assert (np.where(M, P, np.inf).min(1) >= np.where(~M, P, -np.inf).max(1)).all()
    M1, M2 = orc.top_p(P, 0.6), orc.top_p(P, 0.9)
    assert (M2 | ~M1).all()                                # monotone in p


def test_top_p_ties_stable_lower_index_first():
    pr = np.array([[0.25, 0.25, 0.25, 0.25]])
    np.testing.assert_array_equal(orc.top_p(pr, 0.5)[0], [True, True, False, False])
    np.testing.assert_array_equal(orc.top_p(pr, 0.51)[0], [True, True, True, False])


def test_selection_structural_invariants():
    w = wl.small_variant(wl.WORKLOADS["c2_llama_8k"], 2048, 8, 2)
    Qb, Kb, _ = wl.generate(w, n_threads=1)
    sel = orc.prism_select(orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), 64, 96, 128, 0.95)
    N = w.n_blocks
    assert not np.triu(sel.mask, 1).any()                  # no v > u
    assert sel.mask[:, 0, 0].all()                         # row 0 = {0}
    assert (sel.mask.sum(-1) >= 1).all()
    row_ptr, col = orc.mask_to_csr(sel.mask)
    assert row_ptr[-1] == sel.mask.sum() == len(col)
    back = np.zeros_like(sel.mask).reshape(-1, N)
    for r in range(len(row_ptr) - 1):
        c = col[row_ptr[r]:row_ptr[r + 1]]
        assert (np.diff(c) > 0).all()
        back[r, c] = True
    np.testing.assert_array_equal(back.reshape(sel.mask.shape), sel.mask)
    sel1 = orc.prism_select(orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), 64, 96, 128, 1.0)
    np.testing.assert_array_equal(sel1.mask, np.tril(np.ones((N, N), bool))[None].repeat(8, 0))


def test_disabled_band_and_zero_energy():
    rng = np.random.default_rng(1)
    Q = rng.standard_normal((2, 32, 16)); K = rng.standard_normal((1, 32, 16))
    s = orc.prism_select(Q, K, 0, 12, 4, 0.9)
    assert not s.band_masks["high"].any()
    np.testing.assert_array_equal(s.mask, s.band_masks["low"])
    Kz = K.copy(); Kz[..., :8] = 0.0
    s = orc.prism_select(Q, Kz, 8, 12, 4, 0.9)
    tri = np.tril(np.ones((8, 8), bool))
    assert (s.logits["high"][:, tri] == 0.0).all()


def test_temperature_on_coherent_inputs_has_a_closed_form():
    """Every pooled vector the same, with the high dims of Qbar scaled by a and of Kbar by b:
    RMS(Qbar_h) = a q, RMS(Qbar) = q sqrt((d_h a^2 + d - d_h)/d) =: q rq, likewise for K, so
    tau_h = sqrt(d_h/d) (a/rq)(b/rk) and every high-band logit is
    d_h a b q k / (sqrt(d_h) tau_h) = sqrt(d) q k rq rk: the attenuation a, b cancels (the
    restoration the calibration is for) and for a = b = 1 the band logit equals the
    full-spectrum logit sqrt(d) q k.  A wrong prefactor or an inverted RMS ratio fails this."""
    d, d_h, d_l, N = 128, 64, 96, 6
    for a, b, q, k in [(1.0, 1.0, 0.5, 2.0), (0.125, 0.25, 1.5, 0.75), (0.01, 3.0, 1.0, 1.0)]:
        Q = np.full((1, N, d), q); Q[..., :d_h] *= a
        K = np.full((1, N, d), k); K[..., :d_h] *= b
        s = orc.prism_select(Q, K, d_h, d_l, 1, 0.9)
        rq = np.sqrt((d_h * a * a + d - d_h) / d)
        rk = np.sqrt((d_h * b * b + d - d_h) / d)
        tri = np.tril(np.ones((N, N), bool))
        np.testing.assert_allclose(s.tau["high"], np.sqrt(d_h / d) * (a / rq) * (b / rk), rtol=1e-13)
        np.testing.assert_allclose(s.logits["high"][0][tri], np.sqrt(d) * q * k * rq * rk, rtol=1e-12)
        # low band: dims d - d_l .. d-1 hold 32 scaled and 64 unscaled dims
        n_s = d_h - (d - d_l)
        rq_l = np.sqrt((n_s * a * a + d_l - n_s) / d_l)
        rk_l = np.sqrt((n_s * b * b + d_l - n_s) / d_l)
        dot_l = (n_s * a * b + d_l - n_s) * q * k
        want = dot_l / (np.sqrt(d_l) * np.sqrt(d_l / d) * (rq_l / rq) * (rk_l / rk))
        np.testing.assert_allclose(s.logits["low"][0][tri], want, rtol=1e-12)


def test_temperature_on_iid_gaussian_vectors_gives_sqrt_d_over_dz():
    """Independent N(0,1) pooled vectors have the same RMS in every band, so tau_z = sqrt(d_z/d)
    and the band logits q_z.k_z / (d_z / sqrt(d)) have standard deviation sqrt(d/d_z) times that
    of the full-spectrum logits q.k / sqrt(d): 1.414 at d_z = 64, 1.155 at d_z = 96."""
    rng = np.random.default_rng(99)
    d, N = 128, 400
    Q, K = rng.standard_normal((1, N, d)), rng.standard_normal((1, N, d))
    s = orc.prism_select(Q, K, 64, 96, 1, 0.9, causal=False)
    full = (Q[0] @ K[0].T) / np.sqrt(d)
    assert abs(s.logits["high"].std() / full.std() - np.sqrt(2.0)) < 0.02
    assert abs(s.logits["low"].std() / full.std() - np.sqrt(128 / 96)) < 0.02
    np.testing.assert_allclose(s.tau["high"], np.sqrt(0.5), rtol=0.01)
    np.testing.assert_allclose(s.tau["low"], np.sqrt(0.75), rtol=0.01)


def _mask_from_logits(sel, logits, p):
    """Union of the two bands' top-p sets for the given logits (same steps as the oracle)."""
    out = np.zeros_like(sel.mask)
    for z in ("high", "low"):
        for hq in range(out.shape[0]):
            out[hq] |= orc.top_p(orc.softmax_rows(logits[z][hq]), p) & sel.valid
    return out


def test_tolerance_rejects_far_flips_and_accepts_small_score_errors():
    w = wl.small_variant(wl.WORKLOADS["c2_llama_8k"], 4096, 4, 1)
    Qb, Kb, _ = wl.generate(w, n_threads=1)
    p = 0.95
    sel = orc.prism_select(orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), 64, 96, 128, p)
    tol = orc.selection_tolerance(sel, p)
    passes = lambda m: not (tol.must & ~m).any() and not (tol.must_not & m).any()
    assert passes(sel.mask)
    # (a) one block far from the cutoff switched the wrong way is rejected, whichever way
    rng = np.random.default_rng(5)
    for hq in range(4):
        for u in rng.integers(4, 32, size=6):
            far_in = np.argmax(np.where(sel.mask[hq, u], sel.logits["high"][hq, u], -np.inf))
            m = sel.mask.copy(); m[hq, u, far_in] = False
            assert tol.must[hq, u, far_in] and not passes(m)
            cand = ~sel.mask[hq, u] & sel.valid[u]
            if cand.any():
                worst = np.maximum(sel.logits["high"][hq, u], sel.logits["low"][hq, u])
                far_out = np.argmin(np.where(cand, worst, np.inf))
                if tol.must_not[hq, u, far_out]:
                    m = sel.mask.copy(); m[hq, u, far_out] = True
                    assert not passes(m)
    # a block above the diagonal is never acceptable
    m = sel.mask.copy(); m[0, 3, 9] = True
    assert not passes(m)
    # (b) masks recomputed from logits perturbed by up to 5e-4 (half the stated margin) pass
    for seed in range(3):
        r = np.random.default_rng(seed)
        pert = {z: sel.logits[z] + r.uniform(-5e-4, 5e-4, sel.logits[z].shape) for z in ("high", "low")}
        assert passes(_mask_from_logits(sel, pert, p))
    # ... while errors of 2e-2 do not
    r = np.random.default_rng(11)
    pert = {z: sel.logits[z] + r.uniform(-2e-2, 2e-2, sel.logits[z].shape) for z in ("high", "low")}
    assert not passes(_mask_from_logits(sel, pert, p))


def test_tolerance_sets_are_consistent():
    w = wl.small_variant(wl.WORKLOADS["c2_llama_8k"], 4096, 4, 1)
    Qb, Kb, _ = wl.generate(w, n_threads=1)
    sel = orc.prism_select(orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), 64, 96, 128, 0.95)
    tol = orc.selection_tolerance(sel, 0.95)
    assert not (tol.must & tol.must_not).any()
    assert (sel.mask | ~tol.must).all()            # must is a subset of the oracle's mask
    assert not (sel.mask & tol.must_not).any()     # the oracle's own mask passes
    assert tol.dont_care_fraction < 0.005


# --------------------------------------------------------------------------- #
# qualitative behaviour the paper describes (sanity, not parity)
# --------------------------------------------------------------------------- #
def test_planted_slash_is_found_by_high_band_and_calibration_limits_density():
    w = wl.WORKLOADS["c1_2k_slash"]
    Qb, Kb, _ = wl.generate(w, n_threads=1)
    Q, K = orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb)
    sel = orc.prism_select(Q, K, w.d_high, w.d_low, w.block, w.top_p)
    N = w.n_blocks
    # offset 16 < B: the slash lives in blocks u and u-1
    hit = [sel.band_masks["high"][0, u, u] or sel.band_masks["high"][0, u, u - 1]
           for u in range(1, N)]
    assert np.mean(hit) > 0.9
    unc = orc.prism_select(Q, K, w.d_high, w.d_low, w.block, w.top_p, calibrate=False)
    dens = lambda m: m.sum() / (N * (N + 1) / 2)
    assert dens(unc.band_masks["high"]) > dens(sel.band_masks["high"])   # density inflation
