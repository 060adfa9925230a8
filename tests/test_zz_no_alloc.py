"""GPU test of prism_estimate_static, the estimate for callers that cannot allocate: its
scratch is a device array inside the library.  Through the C ABI, on two calls in a row (the
second with a smaller input, so stale scratch contents of the first would show), every output
must equal prism_estimate's bit for bit; a problem beyond the array's size is rejected before
anything is launched."""
import numpy as np
import pytest
import torch

from paper_2602_08426_amd import binding as pb
from paper_2602_08426_amd import workloads as wl
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _both(w):
    Qb, Kb, _ = wl.generate(w)
    qd, kd = pb.bf16_bits_to_device(Qb), pb.bf16_bits_to_device(Kb)
    params = gu.params_for(w)
    ref = gu.gpu_estimate(params, qd, kd)
    mask_bits, row_ptr, col_idx, info = pb.alloc_estimate_outputs(params)
    mask_bits.fill_(-1)
    row_ptr.fill_(-1)
    col_idx.fill_(-1)
    info.fill_(-1)
    pb.prism_estimate_static(params, qd, kd, mask_bits, row_ptr, col_idx, col_idx.numel(), info)
    torch.cuda.synchronize()
    nnz = int(ref["info"][0])
    np.testing.assert_array_equal(info.cpu().numpy(), ref["info"])
    np.testing.assert_array_equal(mask_bits.cpu().numpy().view(np.uint64), ref["words"])
    np.testing.assert_array_equal(row_ptr.cpu().numpy(), ref["row_ptr"])
    np.testing.assert_array_equal(col_idx.cpu().numpy()[:nnz], ref["col_idx"][:nnz])
    return nnz


def test_static_scratch_estimate_equals_workspace_estimate_twice():
    big = wl.small_variant(wl.WORKLOADS["c2_llama_8k"], 128 * 100 + 57, 8, 2)    # ragged, N = 101
    small = wl.small_variant(wl.WORKLOADS["c5_qwen_64k"], 128 * 19, 7, 1)
    for w in (big, small):
        print(f"case {w.name} h={w.n_q_heads}/{w.n_kv_heads} L={w.seq_len}", flush=True)
        assert _both(w) > 0


def test_static_scratch_limit_is_enforced():
    fits = pb.make_params(32, 8, 32768, 128)
    assert pb.prism_estimate_workspace_bytes(fits) <= 16 << 20
    too_big = pb.make_params(32, 8, 65536, 128)
    assert pb.prism_estimate_workspace_bytes(too_big) > 16 << 20
    x = torch.zeros(8, device="cuda")
    with pytest.raises(pb.PrismError) as e:
        pb.prism_estimate_static(too_big, x, x, x, x, x, 1, x)
    assert e.value.status == -5
