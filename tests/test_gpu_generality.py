"""GPU parity for the generality of the boundary: head dims 64 and 256 (the whole path: pooled
vectors, scales, logits, masks, index lists, attention outputs) and packed variable-length
batches (every sequence must come out exactly as the oracle computes it on that sequence alone).
Same bars as the other GPU tests: integer outputs bit-exact, masks exact outside the oracle's
don't-care set, logits within the fp32 tolerance, attention outputs within 2e-2 max-abs and
LSE within 2e-3."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import prism_oracle as orc
from paper_2602_08426_amd import binding as pb
from paper_2602_08426_amd import workloads as wl
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

OUT_TOL = 2e-2
LSE_TOL = 2e-3


def _check_mask(gpu_mask, sel, p, max_dont_care=0.02):
    tol = orc.selection_tolerance(sel, p)
    missing = tol.must & ~gpu_mask
    extra = tol.must_not & gpu_mask
    assert not missing.any(), f"{missing.sum()} must-select blocks missing, first {np.argwhere(missing)[:5]}"
    assert not extra.any(), f"{extra.sum()} forbidden blocks selected, first {np.argwhere(extra)[:5]}"
    assert tol.dont_care_fraction < max_dont_care, tol.dont_care_fraction


def _check_rows(o, l, Q, K, V, mask, B, rows=None):
    """o [h, L, d] float64, l [h, L]: compare the listed (head, q-block) rows with the oracle."""
    ref = orc.block_sparse_attention(Q, K, V, mask, B, rows)
    worst = 0.0
    for (hq, u), (ro, rl) in ref.items():
        sl = slice(u * B, u * B + ro.shape[0])
        err = np.abs(o[hq, sl] - ro).max()
        worst = max(worst, err)
        assert err <= OUT_TOL, f"head {hq} q-block {u}: max-abs {err}"
        fin = np.isfinite(rl)
        assert (np.abs(l[hq, sl][fin] - rl[fin]) <= LSE_TOL).all(), (hq, u)
        assert (l[hq, sl][~fin] == -np.inf).all()
    return worst


@pytest.mark.parametrize("d,d_high,d_low,B,L", [
    (64, 32, 48, 128, 128 * 21 + 50),       # ragged last block
    (64, 32, 48, 64, 64 * 40),
    (64, 64, 64, 128, 128 * 9),             # both bands = the whole head (coarse-attention limit)
    (256, 128, 192, 128, 128 * 19 + 7),     # low band wider than 128 dims: two passes of the score GEMM
    (256, 128, 192, 64, 64 * 37),
    (256, 256, 40, 128, 128 * 12),          # full-width band, and one that is not a multiple of 32
])
def test_head_dims_64_and_256(d, d_high, d_low, B, L):
    print(f"case d={d} bands {d_high}/{d_low} B={B} L={L}", flush=True)
    base = wl.small_variant(wl.WORKLOADS["c3_llama_32k"], L, 4, 2, B)
    w = dataclasses.replace(base, head_dim=d, d_high=d_high, d_low=d_low)
    Qb, Kb, Vb = wl.generate(w)
    assert Qb.shape == (4, L, d)
    qd, kd, vd = (pb.bf16_bits_to_device(x) for x in (Qb, Kb, Vb))
    Q, K, V = orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), orc.bf16_to_f64(Vb)
    sel = orc.prism_select(Q, K, d_high, d_low, B, w.top_p)
    params = gu.params_for(w)
    assert params.head_dim == d

    sc = gu.gpu_block_scores(params, qd, kd)
    assert np.abs(sc["pooled_q"] - sel.q_pooled).max() <= 2e-6 * max(1.0, np.abs(sel.q_pooled).max())
    assert np.abs(sc["pooled_k"] - sel.k_pooled).max() <= 2e-6 * max(1.0, np.abs(sel.k_pooled).max())
    np.testing.assert_allclose(sc["scales"][:, 0], sel.scale["high"], rtol=2e-5)
    np.testing.assert_allclose(sc["scales"][:, 1], sel.scale["low"], rtol=2e-5)
    for z in ("high", "low"):
        got, ref = sc[f"logits_{z}"][:, sel.valid], sel.logits[z][:, sel.valid]
        err = np.abs(got - ref)
        print(f"  logits_{z}: max abs err {err.max():.3g} at |ref| up to {np.abs(ref).max():.3g}", flush=True)
        assert (err <= 2e-5 + 4e-6 * np.abs(ref)).all(), f"{z}: max err {err.max():.3g}"

    res = gu.gpu_estimate(params, qd, kd)
    _check_mask(res["mask"], sel, w.top_p)
    rp_ref, col_ref = orc.mask_to_csr(res["mask"])
    np.testing.assert_array_equal(res["row_ptr"], rp_ref)
    np.testing.assert_array_equal(res["col_idx"][:len(col_ref)], col_ref)
    dens = res["mask"].sum() / sel.valid.sum() / 4
    print(f"  density {dens:.3f}", flush=True)

    _, rp_d, ci_d, _ = res["dev"]
    out, lse = gu.gpu_sparse_attn(params, qd, kd, vd, rp_d, ci_d, int(res["info"][0]))
    o, l = gu.bf16_out_to_f64(out), lse.cpu().numpy().astype(np.float64)
    assert np.isfinite(o).all()
    worst = _check_rows(o, l, Q, K, V, res["mask"], B)
    print(f"  attention on the selected lists: worst max-abs {worst:.4f}", flush=True)

    # dense causal lists through the same kernels against plain causal attention
    _, rp2, ci2, _ = pb.alloc_estimate_outputs(params)
    pb.prism_causal_csr(params, rp2, ci2, ci2.numel())
    out2, lse2 = gu.gpu_sparse_attn(params, qd, kd, vd, rp2, ci2, ci2.numel())
    ref_o, ref_l = orc.dense_causal_attention(Q, K, V)
    assert np.abs(gu.bf16_out_to_f64(out2) - ref_o).max() <= OUT_TOL
    assert np.abs(lse2.cpu().numpy() - ref_l).max() <= LSE_TOL


def _packed_batch(lens, h, hkv, B, d=128, d_high=64, d_low=96):
    """Sequences generated one by one (different seeds), packed along the token axis."""
    parts = []
    for i, L in enumerate(lens):
        w = wl.small_variant(wl.WORKLOADS["c3_llama_32k"], L, h, hkv, B)
        w = dataclasses.replace(w, seed=w.seed + 17 * i, head_dim=d, d_high=d_high, d_low=d_low)
        if L >= 256:
            parts.append(wl.generate(w))
        else:                                  # too short for the planted patterns: plain noise
            rng = np.random.default_rng(w.seed)
            parts.append(tuple(wl.f32_to_bf16_bits(rng.standard_normal((n, L, d)).astype(np.float32))
                               for n in (h, hkv, hkv)))
    Qb, Kb, Vb = (np.ascontiguousarray(np.concatenate([p[j] for p in parts], axis=1)) for j in range(3))
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    return parts, Qb, Kb, Vb, cu, w


@pytest.mark.parametrize("lens,h,hkv,B,d,bands", [
    ([128 * 9, 300, 128 * 20 + 1, 77, 128 * 5], 4, 2, 128, 128, (64, 96)),     # whole-block and ragged sequences mixed
    ([64 * 33, 64, 64 * 7 + 13, 1], 2, 1, 64, 128, (64, 96)),                   # down to a single token
    ([128 * 6, 200, 128 * 11], 4, 2, 128, 64, (32, 48)),
])
def test_varlen_batch_matches_per_sequence_oracle(lens, h, hkv, B, d, bands):
    print(f"case lens={lens} h={h}/{hkv} B={B} d={d}", flush=True)
    parts, Qb, Kb, Vb, cu, w = _packed_batch(lens, h, hkv, B, d, *bands)
    T = int(cu[-1])
    p = w.top_p
    params = pb.make_params(h, hkv, T, B, bands[0], bands[1], p, head_dim=d)
    mo, ro, co = pb.prism_varlen_layout(params, cu)
    Ns = [-(-L // B) for L in lens]
    assert mo[-1] == sum(h * N * (-(-N // 64)) for N in Ns)
    assert ro[-1] == sum(h * N + 1 for N in Ns)
    assert co[-1] == sum(h * N * (N + 1) // 2 for N in Ns)

    qd, kd, vd = (pb.bf16_bits_to_device(x) for x in (Qb, Kb, Vb))
    mask_bits = torch.full((mo[-1],), -1, dtype=torch.int64, device="cuda")
    row_ptr = torch.full((ro[-1],), -7, dtype=torch.int32, device="cuda")
    col_idx = torch.full((co[-1] + 1,), -7, dtype=torch.int32, device="cuda")
    info = torch.full((4 * len(lens),), -7, dtype=torch.int32, device="cuda")
    ws = pb.alloc_workspace(pb.prism_estimate_varlen_workspace_bytes(params, cu))
    pb.prism_estimate_varlen(params, cu, qd, kd, mask_bits, row_ptr, col_idx, info, ws)
    out = torch.full((h, T, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((h, T), float("nan"), dtype=torch.float32, device="cuda")
    ws2 = pb.alloc_workspace(pb.prism_sparse_attn_varlen_workspace_bytes(params, cu))
    pb.prism_sparse_attn_varlen(params, cu, qd, kd, vd, row_ptr, col_idx, out, lse, ws2)
    torch.cuda.synchronize()

    words = mask_bits.cpu().numpy().view(np.uint64)
    rp_all, ci_all, info_all = row_ptr.cpu().numpy(), col_idx.cpu().numpy(), info.cpu().numpy()
    o_all, l_all = gu.bf16_out_to_f64(out), lse.cpu().numpy().astype(np.float64)
    assert np.isfinite(o_all).all() and not np.isnan(l_all).any()
    for s, (L, N) in enumerate(zip(lens, Ns)):
        Qs, Ks, Vs = (orc.bf16_to_f64(x) for x in parts[s])
        sel = orc.prism_select(Qs, Ks, bands[0], bands[1], B, p)
        W = -(-N // 64)
        mask = gu.unpack_mask(words[mo[s]:mo[s + 1]].reshape(h, N, W), N)
        _check_mask(mask, sel, p, max_dont_care=0.05 if N < 16 else 0.02)
        rp_ref, col_ref = orc.mask_to_csr(mask)
        np.testing.assert_array_equal(rp_all[ro[s]:ro[s + 1]], rp_ref)
        np.testing.assert_array_equal(ci_all[co[s]:co[s] + len(col_ref)], col_ref)
        assert info_all[4 * s] == len(col_ref) and info_all[4 * s + 1] == 0
        tok = slice(int(cu[s]), int(cu[s + 1]))
        worst = _check_rows(o_all[:, tok], l_all[:, tok], Qs, Ks, Vs, mask, B)
        print(f"  sequence {s} (L={L}, N={N}): nnz {len(col_ref)}, attention worst max-abs {worst:.4f}", flush=True)

    # the same sequences one call each give bit-identical results
    s = 2
    ps = pb.make_params(h, hkv, lens[s], B, bands[0], bands[1], p, head_dim=d)
    one = gu.gpu_estimate(ps, *(pb.bf16_bits_to_device(parts[s][j]) for j in range(2)))
    N, W = Ns[s], -(-Ns[s] // 64)
    np.testing.assert_array_equal(one["words"].reshape(-1), words[mo[s]:mo[s + 1]])
    np.testing.assert_array_equal(one["row_ptr"], rp_all[ro[s]:ro[s + 1]])


@pytest.mark.parametrize("d,B", [(64, 128), (256, 64)])
def test_other_head_dims_bidirectional_and_slice_bands(d, B):
    """Bidirectional selection and attention, bands given as two slices each, at head dims 64 / 256."""
    L = B * 18
    base = wl.small_variant(wl.WORKLOADS["c3_llama_32k"], L, 4, 2, B)
    w = dataclasses.replace(base, head_dim=d, d_high=d // 2, d_low=3 * d // 4)
    Qb, Kb, Vb = wl.generate(w)
    qd, kd, vd = (pb.bf16_bits_to_device(x) for x in (Qb, Kb, Vb))
    Q, K, V = orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), orc.bf16_to_f64(Vb)
    high = [(0, d // 8), (d // 2, d // 8)]                   # two slices: dims [0, d/8) and [d/2, 5d/8)
    low = [(d // 4, d // 4), (3 * d // 4, d // 4)]
    p = 0.9
    sel = orc.prism_select(Q, K, 0, 0, B, p, causal=False, bands={"high": high, "low": low})
    params = gu.params_for(w, top_p=p, flags=pb.PRISM_FLAG_BIDIRECTIONAL)
    res = gu.gpu_estimate(params, qd, kd, bands=pb.make_bands(high, low))
    _check_mask(res["mask"], sel, p)
    assert np.triu(res["mask"], 1).any()
    _, rp_d, ci_d, _ = res["dev"]
    out, lse = gu.gpu_sparse_attn(params, qd, kd, vd, rp_d, ci_d, int(res["info"][0]))
    o, l = gu.bf16_out_to_f64(out), lse.cpu().numpy().astype(np.float64)
    ref = orc.block_sparse_attention(Q, K, V, res["mask"], B, None, causal=False)
    for (hq, u), (ro, rl) in ref.items():
        sl = slice(u * B, u * B + ro.shape[0])
        assert np.abs(o[hq, sl] - ro).max() <= OUT_TOL, (hq, u)
        fin = np.isfinite(rl)
        assert (np.abs(l[hq, sl][fin] - rl[fin]) <= LSE_TOL).all(), (hq, u)


def test_varlen_bidirectional_batch():
    lens, h, hkv, B, d = [128 * 5, 128 * 3 + 50, 128 * 8], 4, 2, 128, 128
    parts, Qb, Kb, Vb, cu, w = _packed_batch(lens, h, hkv, B, d, 64, 96)
    T, p = int(cu[-1]), w.top_p
    params = pb.make_params(h, hkv, T, B, 64, 96, p, flags=pb.PRISM_FLAG_BIDIRECTIONAL, head_dim=d)
    mo, ro, co = pb.prism_varlen_layout(params, cu)
    Ns = [-(-L // B) for L in lens]
    assert co[-1] == sum(h * N * N for N in Ns)
    qd, kd, vd = (pb.bf16_bits_to_device(x) for x in (Qb, Kb, Vb))
    mask_bits = torch.zeros((mo[-1],), dtype=torch.int64, device="cuda")
    row_ptr = torch.zeros((ro[-1],), dtype=torch.int32, device="cuda")
    col_idx = torch.zeros((co[-1] + 1,), dtype=torch.int32, device="cuda")
    info = torch.zeros((4 * len(lens),), dtype=torch.int32, device="cuda")
    pb.prism_estimate_varlen(params, cu, qd, kd, mask_bits, row_ptr, col_idx, info,
                             pb.alloc_workspace(pb.prism_estimate_varlen_workspace_bytes(params, cu)))
    out = torch.full((h, T, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((h, T), float("nan"), dtype=torch.float32, device="cuda")
    pb.prism_sparse_attn_varlen(params, cu, qd, kd, vd, row_ptr, col_idx, out, lse,
                                pb.alloc_workspace(pb.prism_sparse_attn_varlen_workspace_bytes(params, cu)))
    torch.cuda.synchronize()
    words = mask_bits.cpu().numpy().view(np.uint64)
    o_all, l_all = gu.bf16_out_to_f64(out), lse.cpu().numpy().astype(np.float64)
    for s, (L, N) in enumerate(zip(lens, Ns)):
        Qs, Ks, Vs = (orc.bf16_to_f64(x) for x in parts[s])
        sel = orc.prism_select(Qs, Ks, 64, 96, B, p, causal=False)
        mask = gu.unpack_mask(words[mo[s]:mo[s + 1]].reshape(h, N, -(-N // 64)), N)
        _check_mask(mask, sel, p, max_dont_care=0.05)
        ref = orc.block_sparse_attention(Qs, Ks, Vs, mask, B, None, causal=False)
        for (hq, u), (ro_, rl) in ref.items():
            sl = slice(int(cu[s]) + u * B, int(cu[s]) + u * B + ro_.shape[0])
            assert np.abs(o_all[hq, sl] - ro_).max() <= OUT_TOL, (s, hq, u)
            fin = np.isfinite(rl)
            assert (np.abs(l_all[hq, sl][fin] - rl[fin]) <= LSE_TOL).all(), (s, hq, u)
