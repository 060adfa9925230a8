"""GPU parity of prism_rope_estimate (estimation fused with the RoPE producer) against the oracle.

Bars: the rotated tensors equal the fp64 oracle rotation rounded to bf16 except where the fp32
evaluation of cos / sin moves a value across a rounding boundary (fewer than 2e-3 of the elements;
error at most half a bf16 step plus 2e-6 of the pair's magnitude); the masks are those of the oracle's selection on the tensors the
GPU wrote (exact outside the 1e-3 cutoff margin) and bit for bit those of prism_estimate on them.
"""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import prism_oracle as orc
from paper_2602_08426_amd import binding as pb
from paper_2602_08426_amd import workloads as wl
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

YARN = (32768, 4.0, 1.0, 32.0)      # App. "Compatibility with YaRN": native length, s, alpha, beta


def _run(w, position_offset=0, in_place=False):
    Qb, Kb, _ = wl.generate(w, rotate=False)
    q_in, k_in = pb.bf16_bits_to_device(Qb), pb.bf16_bits_to_device(Kb)
    q_out = q_in if in_place else torch.full_like(q_in, float("nan"))
    k_out = k_in if in_place else torch.full_like(k_in, float("nan"))
    params = gu.params_for(w)
    rope = pb.make_rope(w.rope_base, position_offset, *(w.yarn if w.yarn else (0, 1.0, 1.0, 32.0)))
    mask_bits, row_ptr, col_idx, info = pb.alloc_estimate_outputs(params)
    ws = pb.alloc_workspace(pb.prism_estimate_workspace_bytes(params))
    pb.prism_rope_estimate(params, rope, None, q_in, k_in, q_out, k_out, mask_bits, row_ptr, col_idx,
                           col_idx.numel(), info, ws)
    torch.cuda.synchronize()
    return Qb, Kb, q_out, k_out, params, (mask_bits, row_ptr, col_idx, info)


def _check_rotation(w, pre_bits, out_dev, position_offset):
    theta = orc.rope_frequencies(w.head_dim, w.rope_base, yarn=w.yarn)
    ref = orc.apply_rope(orc.bf16_to_f64(pre_bits), theta, position_offset)
    ref_bits = orc.f64_to_bf16_bits(ref)
    got_bits = out_dev.view(torch.int16).cpu().numpy().view(np.uint16)
    diff = got_bits != ref_bits
    frac = diff.mean()
    assert frac < 2e-3, f"{frac:.2e} of the rotated elements differ from the rounded oracle"
    # error budget: half a bf16 step of rounding plus the fp32 evaluation of the rotation, which is
    # relative to the magnitude of the pair (a component can be small by cancellation)
    got = orc.bf16_to_f64(got_bits)
    pre = orc.bf16_to_f64(pre_bits)
    pair = np.repeat(np.hypot(pre[..., 0::2], pre[..., 1::2]), 2, axis=-1)
    err = np.abs(got - ref)
    assert (err <= np.abs(ref) * 2.0 ** -8 + 2e-6 * pair + 1e-30).all()
    # away from cancellation a differing element is the neighbouring bf16 value
    big = diff & (np.abs(ref) > 1e-2 * pair)
    step = np.abs(got_bits[big].astype(np.int32) - ref_bits[big].astype(np.int32))
    assert (step == 1).all()
    return got_bits


@pytest.mark.parametrize("L,h,hkv,B,yarn,offset", [
    (2048, 8, 2, 128, None, 0),
    (128 * 9 + 40, 4, 2, 128, None, 1000),          # ragged last block, positions shifted
    (2048, 4, 1, 64, YARN, 0),
    (4096, 8, 2, 128, YARN, 126976),                 # positions up to 131071 (the 128K range)
])
def test_fused_rope_matches_oracle_rotation_and_selection(L, h, hkv, B, yarn, offset):
    print(f"case L={L} h={h}/{hkv} B={B} yarn={yarn} offset={offset}", flush=True)
    w = dataclasses.replace(wl.small_variant(wl.WORKLOADS["c5_qwen_64k"], L, h, hkv), block=B, yarn=yarn)
    Qb, Kb, q_out, k_out, params, outs = _run(w, offset)
    q_bits = _check_rotation(w, Qb, q_out, offset)
    k_bits = _check_rotation(w, Kb, k_out, offset)
    N = params.n_blocks
    mask = gu.unpack_mask(outs[0].cpu().numpy().view(np.uint64), N)
    # the selection on the tensors the GPU wrote
    sel = orc.prism_select(orc.bf16_to_f64(q_bits), orc.bf16_to_f64(k_bits), w.d_high, w.d_low, B, w.top_p)
    tol = orc.selection_tolerance(sel, w.top_p)
    assert not (tol.must & ~mask).any() and not (tol.must_not & mask).any()
    # ... and bit for bit what the unfused call gives on them
    plain = gu.gpu_estimate(params, q_out, k_out)
    assert np.array_equal(plain["words"], outs[0].cpu().numpy().view(np.uint64))
    assert np.array_equal(plain["row_ptr"], outs[1].cpu().numpy())
    nnz = int(outs[3][0].item())
    assert np.array_equal(plain["col_idx"][:nnz], outs[2].cpu().numpy()[:nnz])


@pytest.mark.parametrize("d,d_high,d_low,B,L,offset", [
    (64, 32, 48, 128, 128 * 11 + 9, 0),
    (64, 32, 48, 64, 2048, 4000),
    (256, 128, 192, 128, 128 * 10, 0),
    (256, 128, 192, 64, 64 * 21 + 5, 120000),       # sixteen rows per thread: the longest fp32 recurrence
])
def test_fused_rope_other_head_dims(d, d_high, d_low, B, L, offset):
    print(f"case d={d} B={B} L={L} offset={offset}", flush=True)
    base = wl.small_variant(wl.WORKLOADS["c3_llama_32k"], L, 4, 2, B)
    w = dataclasses.replace(base, head_dim=d, d_high=d_high, d_low=d_low)
    Qb, Kb, q_out, k_out, params, outs = _run(w, offset)
    assert params.head_dim == d
    q_bits = _check_rotation(w, Qb, q_out, offset)
    k_bits = _check_rotation(w, Kb, k_out, offset)
    N = params.n_blocks
    mask = gu.unpack_mask(outs[0].cpu().numpy().view(np.uint64), N)
    sel = orc.prism_select(orc.bf16_to_f64(q_bits), orc.bf16_to_f64(k_bits), d_high, d_low, B, w.top_p)
    tol = orc.selection_tolerance(sel, w.top_p)
    assert not (tol.must & ~mask).any() and not (tol.must_not & mask).any()
    plain = gu.gpu_estimate(params, q_out, k_out)
    assert np.array_equal(plain["words"], outs[0].cpu().numpy().view(np.uint64))


def test_fused_rope_in_place_equals_out_of_place():
    w = wl.small_variant(wl.WORKLOADS["c2_llama_8k"], 2048, 8, 2)
    _, _, q1, k1, _, o1 = _run(w, 17, in_place=False)
    _, _, q2, k2, _, o2 = _run(w, 17, in_place=True)
    assert torch.equal(q1.view(torch.int16), q2.view(torch.int16))
    assert torch.equal(k1.view(torch.int16), k2.view(torch.int16))
    assert torch.equal(o1[0], o2[0])


def test_selection_parity_holds_under_yarn_frequencies():
    """The GPU path knows nothing of the frequencies: inputs generated with the YaRN-scaled ladder go
    through plain prism_estimate and must match the oracle like any other input."""
    w = dataclasses.replace(wl.small_variant(wl.WORKLOADS["c5_qwen_64k"], 8192, 7, 1), yarn=YARN)
    Qb, Kb, _ = wl.generate(w)
    params = gu.params_for(w)
    res = gu.gpu_estimate(params, pb.bf16_bits_to_device(Qb), pb.bf16_bits_to_device(Kb))
    sel = orc.prism_select(orc.bf16_to_f64(Qb), orc.bf16_to_f64(Kb), w.d_high, w.d_low, w.block, w.top_p)
    tol = orc.selection_tolerance(sel, w.top_p)
    assert not (tol.must & ~res["mask"]).any() and not (tol.must_not & res["mask"]).any()
    assert tol.dont_care_fraction < 0.02
