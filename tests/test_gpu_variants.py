"""GPU parity for the variants beyond the contiguous-band causal path: bands given as slice
lists (axis-wise bands of App. "HunyuanVideo Spectral Configuration", half-split RoPE storage,
widths that are not multiples of 32), bidirectional selection and attention, forced blocks,
and a batch folded into the head axis.  Same bars as the other GPU tests: integer outputs
bit-exact, masks exact outside the oracle's don't-care set, logits within the fp32 tolerance,
attention outputs within 2e-2 max-abs."""
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

# three axis subspaces [16, 56, 56]: first 8 / 32 / 32 dims and last 16 / 36 / 36 dims
AXIS_HIGH = [(0, 8), (16, 32), (72, 32)]
AXIS_LOW = [(0, 16), (36, 36), (92, 36)]


def _check_mask(gpu_mask, sel, p, max_dont_care):
    tol = orc.selection_tolerance(sel, p)
    missing = tol.must & ~gpu_mask
    extra = tol.must_not & gpu_mask
    assert not missing.any(), f"{missing.sum()} must-select blocks missing, first {np.argwhere(missing)[:5]}"
    assert not extra.any(), f"{extra.sum()} forbidden blocks selected, first {np.argwhere(extra)[:5]}"
    assert tol.dont_care_fraction < max_dont_care, tol.dont_care_fraction


def _check_csr(res):
    rp_ref, col_ref = orc.mask_to_csr(res["mask"])
    np.testing.assert_array_equal(res["row_ptr"], rp_ref)
    np.testing.assert_array_equal(res["col_idx"][:len(col_ref)], col_ref)
    assert res["info"][0] == len(col_ref) and res["info"][1] == 0


def _check_logits(sc, sel, valid):
    for z in ("high", "low"):
        got, ref = sc[f"logits_{z}"][:, valid], sel.logits[z][:, valid]
        err = np.abs(got - ref)
        bad = int((err > 2e-5 + 4e-6 * np.abs(ref)).sum())
        print(f"  logits_{z}: max abs err {err.max():.3g} at |ref| up to {np.abs(ref).max():.3g}", flush=True)
        assert bad == 0, f"{z}: {bad} logits off, max err {err.max():.3g}"
        assert np.isnan(sc[f"logits_{z}"][:, ~valid]).all()


@pytest.mark.parametrize("L,h,hkv,B,bidir", [
    (128 * 40, 4, 2, 128, True),       # ragged strip and column tile, bidirectional
    (64 * 130, 2, 1, 64, True),        # three 64-column chunks per row
    (128 * 40, 4, 2, 128, False),      # the same bands under the causal restriction
])
def test_axiswise_bands(L, h, hkv, B, bidir):
    print(f"case L={L} h={h}/{hkv} B={B} bidirectional={bidir}", flush=True)
    w = wl.small_variant(wl.WORKLOADS["c3_llama_32k"], L, h, hkv, B)
    Qb, Kb, _ = wl.generate(w)
    qd, kd = pb.bf16_bits_to_device(Qb), pb.bf16_bits_to_device(Kb)
    p = 0.9
    bands = {"high": AXIS_HIGH, "low": AXIS_LOW}
    sel = orc.prism_select(orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), 0, 0, B, p, causal=not bidir,
                           bands=bands)
    params = gu.params_for(w, top_p=p, flags=pb.PRISM_FLAG_BIDIRECTIONAL if bidir else 0)
    pbands = pb.make_bands(AXIS_HIGH, AXIS_LOW)
    sc = gu.gpu_block_scores(params, qd, kd, bands=pbands)
    np.testing.assert_allclose(sc["scales"][:, 0], sel.scale["high"], rtol=2e-5)
    np.testing.assert_allclose(sc["scales"][:, 1], sel.scale["low"], rtol=2e-5)
    _check_logits(sc, sel, sel.valid)
    res = gu.gpu_estimate(params, qd, kd, bands=pbands)
    _check_mask(res["mask"], sel, p, 0.02)
    _check_csr(res)
    if bidir:
        assert np.triu(res["mask"], 1).any()              # blocks above the diagonal are in play
    else:
        assert not np.triu(res["mask"], 1).any()


def test_half_split_bands_on_permuted_dims_and_odd_widths():
    """RoPE stored as pairs (j, j + d/2): the two-slice bands on the permuted tensors give the
    logits of the contiguous bands on the original ones.  Also contiguous bands whose width is
    not a multiple of 32 (zero-padded k-step)."""
    w = wl.small_variant(wl.WORKLOADS["c3_llama_32k"], 128 * 24, 4, 2)
    Qb, Kb, _ = wl.generate(w)
    to_half = np.concatenate([np.arange(0, 128, 2), np.arange(1, 128, 2)])
    Qp, Kp = np.ascontiguousarray(Qb[:, :, to_half]), np.ascontiguousarray(Kb[:, :, to_half])
    sel = orc.prism_select(orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), w.d_high, w.d_low, w.block, w.top_p)
    params = gu.params_for(w)
    half = pb.make_bands([(0, w.d_high // 2), (64, w.d_high // 2)],
                         [(64 - w.d_low // 2, w.d_low // 2), (128 - w.d_low // 2, w.d_low // 2)])
    qd, kd = pb.bf16_bits_to_device(Qp), pb.bf16_bits_to_device(Kp)
    sc = gu.gpu_block_scores(params, qd, kd, bands=half)
    _check_logits(sc, sel, sel.valid)
    res = gu.gpu_estimate(params, qd, kd, bands=half)
    _check_mask(res["mask"], sel, w.top_p, 0.02)
    _check_csr(res)

    for d_h, d_l in ((48, 72), (8, 120), (100, 1)):
        print(f"  widths {d_h}/{d_l}", flush=True)
        sel2 = orc.prism_select(orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), d_h, d_l, w.block, w.top_p)
        p2 = gu.params_for(w, d_high=d_h, d_low=d_l)
        qo, ko = pb.bf16_bits_to_device(Qb), pb.bf16_bits_to_device(Kb)
        sc2 = gu.gpu_block_scores(p2, qo, ko)
        _check_logits(sc2, sel2, sel2.valid)
        res2 = gu.gpu_estimate(p2, qo, ko)
        _check_mask(res2["mask"], sel2, w.top_p, 0.02)
        _check_csr(res2)


def test_forced_diagonal_and_sink_blocks():
    w = wl.small_variant(wl.WORKLOADS["c3_llama_32k"], 128 * 70, 4, 2)
    Qb, Kb, _ = wl.generate(w)
    qd, kd = pb.bf16_bits_to_device(Qb), pb.bf16_bits_to_device(Kb)
    p = 0.5
    base = gu.gpu_estimate(gu.params_for(w, top_p=p), qd, kd)
    N = w.n_blocks
    eye = np.eye(N, dtype=bool)[None]
    sink = np.zeros((1, N, N), bool); sink[:, :, 0] = True
    for flags, extra in ((pb.PRISM_FLAG_FORCE_DIAGONAL, eye), (pb.PRISM_FLAG_FORCE_SINK, sink),
                         (pb.PRISM_FLAG_FORCE_DIAGONAL | pb.PRISM_FLAG_FORCE_SINK, eye | sink)):
        res = gu.gpu_estimate(gu.params_for(w, top_p=p, flags=flags), qd, kd)
        np.testing.assert_array_equal(res["mask"], base["mask"] | extra)
        _check_csr(res)
    assert (~base["mask"] & eye).any()            # the option changed something at this p
    sel = orc.prism_select(orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), w.d_high, w.d_low, w.block, p,
                           force_diagonal=True, force_sink=True)
    _check_mask(res["mask"], sel, p, 0.02)


def _compare_rows(params, out, lse, Q, K, V, mask, causal):
    B = params.block
    ref = orc.block_sparse_attention(Q, K, V, mask, B, None, causal=causal)
    o = gu.bf16_out_to_f64(out)
    l = lse.cpu().numpy().astype(np.float64)
    for (hq, u), (ro, rl) in ref.items():
        sl = slice(u * B, (u + 1) * B)
        err = np.abs(o[hq, sl] - ro).max()
        assert err <= OUT_TOL, f"head {hq} q-block {u}: max-abs {err}"
        fin = np.isfinite(rl)
        assert (np.abs(l[hq, sl][fin] - rl[fin]) <= LSE_TOL).all(), (hq, u)
        assert (l[hq, sl][~fin] == -np.inf).all()


@pytest.mark.parametrize("h,hkv,L,B,density,seed", [
    (4, 2, 128 * 7, 128, 0.4, 11),
    (2, 1, 64 * 9, 64, 0.5, 12),
    (1, 1, 128, 128, 1.0, 13),
])
def test_bidirectional_attention_matches_oracle(h, hkv, L, B, density, seed):
    print(f"case h={h}/{hkv} L={L} B={B} density={density}", flush=True)
    rng = np.random.default_rng(seed)
    Qb = wl.f32_to_bf16_bits(rng.standard_normal((h, L, 128)).astype(np.float32) * 1.5)
    Kb = wl.f32_to_bf16_bits(rng.standard_normal((hkv, L, 128)).astype(np.float32) * 1.5)
    Vb = wl.f32_to_bf16_bits(rng.standard_normal((hkv, L, 128)).astype(np.float32))
    N = L // B
    mask = rng.random((h, N, N)) < density
    if N > 3:
        mask[:, 2, :] = False                          # empty rows
        mask[0, 1, :] = False
        mask[0, 1, N - 1] = True                       # only a block above the diagonal
    params = pb.make_params(h, hkv, L, B, flags=pb.PRISM_FLAG_BIDIRECTIONAL)
    rp, ci = orc.mask_to_csr(mask)
    ci = ci.copy()
    rp_d, ci_d, cnt = gu.csr_to_device(rp, ci)
    qd, kd, vd = (pb.bf16_bits_to_device(x) for x in (Qb, Kb, Vb))
    out, lse = gu.gpu_sparse_attn(params, qd, kd, vd, rp_d, ci_d, cnt)
    Q, K, V = orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), orc.bf16_to_f64(Vb)
    _compare_rows(params, out, lse, Q, K, V, mask, causal=False)
    # the same lists under the causal flag drop everything above the diagonal
    pc = pb.make_params(h, hkv, L, B)
    out_c, lse_c = gu.gpu_sparse_attn(pc, qd, kd, vd, rp_d, ci_d, cnt)
    _compare_rows(pc, out_c, lse_c, Q, K, V, np.tril(mask), causal=True)


def test_bidirectional_dense_lists_and_out_of_range_entries():
    rng = np.random.default_rng(14)
    h, hkv, L, B = 4, 2, 128 * 6, 128
    N = L // B
    Qb = wl.f32_to_bf16_bits(rng.standard_normal((h, L, 128)).astype(np.float32))
    Kb = wl.f32_to_bf16_bits(rng.standard_normal((hkv, L, 128)).astype(np.float32))
    Vb = wl.f32_to_bf16_bits(rng.standard_normal((hkv, L, 128)).astype(np.float32))
    params = pb.make_params(h, hkv, L, B, flags=pb.PRISM_FLAG_BIDIRECTIONAL)
    _, row_ptr, col_idx, _ = pb.alloc_estimate_outputs(params)
    assert col_idx.numel() == h * N * N
    pb.prism_dense_csr(params, row_ptr, col_idx, col_idx.numel())
    torch.cuda.synchronize()
    np.testing.assert_array_equal(row_ptr.cpu().numpy(), np.arange(h * N + 1) * N)
    np.testing.assert_array_equal(col_idx.cpu().numpy(), np.tile(np.arange(N), h * N))
    qd, kd, vd = (pb.bf16_bits_to_device(x) for x in (Qb, Kb, Vb))
    out, lse = gu.gpu_sparse_attn(params, qd, kd, vd, row_ptr, col_idx, col_idx.numel())
    ref_o, ref_l = orc.dense_full_attention(orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), orc.bf16_to_f64(Vb))
    assert np.abs(gu.bf16_out_to_f64(out) - ref_o).max() <= OUT_TOL
    assert np.abs(lse.cpu().numpy() - ref_l).max() <= LSE_TOL
    # entries outside [0, N) are skipped
    rows = [[0, 5, 6, -3], [99, 1, 4]] + [[u] for u in range(2, h * N)]
    rp = np.zeros(h * N + 1, np.int32); rp[1:] = np.cumsum([len(r) for r in rows])
    ci = np.concatenate(rows).astype(np.int32)
    mask = np.zeros((h, N, N), bool)
    for r, lst in enumerate(rows):
        for v in lst:
            if 0 <= v < N:
                mask[r // N, r % N, v] = True
    rp_d, ci_d, cnt = gu.csr_to_device(rp, ci)
    out2, lse2 = gu.gpu_sparse_attn(params, qd, kd, vd, rp_d, ci_d, cnt)
    _compare_rows(params, out2, lse2, orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), orc.bf16_to_f64(Vb),
                  mask, causal=False)


def test_batch_folded_into_heads_equals_separate_calls():
    """Two batch items of a 4/2-head layer as one 8/4-head call: identical bits."""
    w = wl.small_variant(wl.WORKLOADS["c2_llama_8k"], 128 * 12, 4, 2)
    items = []
    for seed_shift in (0, 7):
        wi = dataclasses.replace(w, seed=w.seed + seed_shift)
        items.append(wl.generate(wi))
    fold = [np.concatenate([it[i] for it in items], axis=0) for i in range(3)]
    pf = gu.params_for(w, n_q_heads=8, n_kv_heads=4)
    ps = gu.params_for(w)

    def run(params, Qb, Kb, Vb):
        qd, kd, vd = (pb.bf16_bits_to_device(x) for x in (Qb, Kb, Vb))
        res = gu.gpu_estimate(params, qd, kd)
        _, rp, ci, _ = res["dev"]
        out, lse = gu.gpu_sparse_attn(params, qd, kd, vd, rp, ci, int(res["info"][0]))
        return res["mask"], pb.device_bf16_to_bits(out), lse.cpu().numpy()

    mf, of, lf = run(pf, *fold)
    for b, it in enumerate(items):
        ms, os_, ls = run(ps, *it)
        np.testing.assert_array_equal(mf[4 * b:4 * b + 4], ms)
        np.testing.assert_array_equal(of[4 * b:4 * b + 4], os_)
        np.testing.assert_array_equal(lf[4 * b:4 * b + 4], ls)


def _ragged_inputs(L, h, hkv, B, name="c3_llama_32k"):
    """Structured workload generated for whole blocks, truncated to L tokens."""
    Lfull = -(-L // B) * B
    w = wl.small_variant(wl.WORKLOADS[name], Lfull, h, hkv, B)
    Qb, Kb, Vb = wl.generate(w)
    return w, tuple(np.ascontiguousarray(x[:, :L]) for x in (Qb, Kb, Vb))


@pytest.mark.parametrize("L,h,hkv,B,flags", [
    (128 * 9 + 37, 4, 2, 128, 0),
    (64 * 20 + 1, 2, 1, 64, 0),                               # a single token in the last block
    (128 * 5 + 100, 4, 2, 128, pb.PRISM_FLAG_BIDIRECTIONAL),
    (90, 2, 2, 128, 0),                                       # one ragged block in all
])
def test_ragged_last_block(L, h, hkv, B, flags):
    """N = ceil(L / B): the last block is pooled over the tokens it holds, its missing keys
    are invisible and its missing queries are not written."""
    print(f"case L={L} h={h}/{hkv} B={B} flags={flags}", flush=True)
    w, (Qb, Kb, Vb) = _ragged_inputs(L, h, hkv, B)
    causal = not (flags & pb.PRISM_FLAG_BIDIRECTIONAL)
    N = -(-L // B)
    p = 0.9
    Q, K, V = orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), orc.bf16_to_f64(Vb)
    sel = orc.prism_select(Q, K, w.d_high, w.d_low, B, p, causal=causal)
    params = pb.make_params(h, hkv, L, B, w.d_high, w.d_low, p, flags)
    assert params.n_blocks == N == sel.mask.shape[1]
    qd, kd, vd = (pb.bf16_bits_to_device(x) for x in (Qb, Kb, Vb))
    sc = gu.gpu_block_scores(params, qd, kd)
    np.testing.assert_allclose(sc["pooled_q"], sel.q_pooled, rtol=2e-6, atol=2e-6)
    np.testing.assert_allclose(sc["pooled_k"], sel.k_pooled, rtol=2e-6, atol=2e-6)
    _check_logits(sc, sel, sel.valid)
    res = gu.gpu_estimate(params, qd, kd)
    _check_mask(res["mask"], sel, p, 0.02)
    _check_csr(res)
    # attention on the GPU's own lists, plus the dense lists
    _, rp, ci, _ = res["dev"]
    h_, L_ = params.n_q_heads, params.seq_len
    guard = 64                                               # rows behind the output must stay untouched
    out = torch.full((h_ * L_ + guard, 128), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((h_ * L_ + guard,), float("nan"), dtype=torch.float32, device="cuda")
    ws = pb.alloc_workspace(pb.prism_sparse_attn_workspace_bytes(params))
    pb.prism_sparse_attn(params, qd, kd, vd, rp, ci, int(res["info"][0]), out[:h_ * L_].view(h_, L_, 128),
                         lse[:h_ * L_].view(h_, L_), ws)
    torch.cuda.synchronize()
    assert torch.isnan(out[h_ * L_:].float()).all() and torch.isnan(lse[h_ * L_:]).all()
    _compare_rows(params, out[:h_ * L_].view(h_, L_, 128), lse[:h_ * L_].view(h_, L_), Q, K, V,
                  res["mask"], causal)
    _, rpd, cid, _ = pb.alloc_estimate_outputs(params)
    pb.prism_dense_csr(params, rpd, cid, cid.numel())
    out_d, lse_d = gu.gpu_sparse_attn(params, qd, kd, vd, rpd, cid, cid.numel())
    ref_o, ref_l = (orc.dense_causal_attention(Q, K, V) if causal else orc.dense_full_attention(Q, K, V))
    assert np.abs(gu.bf16_out_to_f64(out_d) - ref_o).max() <= OUT_TOL
    assert np.abs(lse_d.cpu().numpy() - ref_l).max() <= LSE_TOL


def test_stream_only_flag_runs_and_leaves_later_calls_exact():
    """PRISM_FLAG_STREAM_ONLY is a measurement aid: the call must complete (same tile copies and
    queue traffic, no arithmetic) and a following ordinary call through the same workspace must
    give bitwise the result it gave before."""
    rng = np.random.default_rng(21)
    h, hkv, L, B = 4, 2, 128 * 9, 128
    Qb = wl.f32_to_bf16_bits(rng.standard_normal((h, L, 128)).astype(np.float32))
    Kb = wl.f32_to_bf16_bits(rng.standard_normal((hkv, L, 128)).astype(np.float32))
    Vb = wl.f32_to_bf16_bits(rng.standard_normal((hkv, L, 128)).astype(np.float32))
    N = L // B
    mask = np.tril(rng.random((h, N, N)) < 0.5)
    rp, ci = orc.mask_to_csr(mask)
    rp_d, ci_d, cnt = gu.csr_to_device(rp, ci)
    qd, kd, vd = (pb.bf16_bits_to_device(x) for x in (Qb, Kb, Vb))
    params = pb.make_params(h, hkv, L, B)
    ws = pb.alloc_workspace(pb.prism_sparse_attn_workspace_bytes(params))
    out0 = torch.empty_like(qd)
    pb.prism_sparse_attn(params, qd, kd, vd, rp_d, ci_d, cnt, out0, None, ws)
    torch.cuda.synchronize()
    p_stream = pb.make_params(h, hkv, L, B, flags=pb.PRISM_FLAG_STREAM_ONLY)
    scratch = torch.empty_like(qd)
    pb.prism_sparse_attn(p_stream, qd, kd, vd, rp_d, ci_d, cnt, scratch, None, ws)
    torch.cuda.synchronize()
    out1 = torch.empty_like(qd)
    pb.prism_sparse_attn(params, qd, kd, vd, rp_d, ci_d, cnt, out1, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(out0.view(torch.int16), out1.view(torch.int16))


def test_hip_graph_replays_match_eager_calls():
    """No entry point allocates, synchronises or records a memset, so a caller can capture
    estimate -> V image -> attention in a HIP graph.  Every replay (with eager work and
    synchronisations between them, and new input values in the captured buffers) must give
    bitwise what the eager calls give on the same inputs."""
    w = wl.small_variant(wl.WORKLOADS["c2_llama_8k"], 2048, 8, 2)
    params = gu.params_for(w)
    inputs = []
    for seed in (w.seed, w.seed + 1, w.seed + 2):
        Qb, Kb, Vb = wl.generate(dataclasses.replace(w, seed=seed))
        inputs.append(tuple(pb.bf16_bits_to_device(x) for x in (Qb, Kb, Vb)))
    q, k, v = (torch.empty_like(x) for x in inputs[0])
    mask_bits, row_ptr, col_idx, info = pb.alloc_estimate_outputs(params)
    cap = col_idx.numel()
    ws_e = pb.alloc_workspace(pb.prism_estimate_workspace_bytes(params))
    ws_a = pb.alloc_workspace(pb.prism_sparse_attn_workspace_bytes(params))
    out = torch.empty_like(q)
    lse = torch.empty((w.n_q_heads, w.seq_len), dtype=torch.float32, device="cuda")

    def run():
        pb.prism_estimate(params, q, k, mask_bits, row_ptr, col_idx, cap, info, ws_e)
        pb.prism_v_image(params, v, ws_a)
        pb.prism_sparse_attn_pre(params, q, k, ws_a, row_ptr, col_idx, cap, out, lse)

    eager = []
    for qi, ki, vi in inputs:
        q.copy_(qi); k.copy_(ki); v.copy_(vi)
        run()
        torch.cuda.synchronize()
        eager.append((out.clone(), lse.clone(), mask_bits.clone(), int(info[0].item())))

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for rep in range(2):
        for (qi, ki, vi), (o_ref, l_ref, m_ref, nnz_ref) in zip(inputs, eager):
            q.copy_(qi); k.copy_(ki); v.copy_(vi)
            out.zero_(); lse.zero_(); mask_bits.zero_()        # eager work between the replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert int(info[0].item()) == nnz_ref
            assert torch.equal(mask_bits, m_ref)
            assert torch.equal(out.view(torch.int16), o_ref.view(torch.int16))
            assert torch.equal(lse, l_ref)
