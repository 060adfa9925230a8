"""Host-side checks of the C ABI (no GPU): the library loads, exports every symbol that
include/prism.h declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

from paper_2602_08426_amd import binding as pb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "prism.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(pb.library_path()):
        from paper_2602_08426_amd.build import build_library
        build_library()
    return pb._load()


def _declared():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(prism_[a-z_]+)\s*\(", src)))


def test_exports_every_declared_symbol(lib):
    names = _declared()
    assert set(names) == set(pb.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_status_strings(lib):
    assert pb.prism_version() >= 100
    assert pb.prism_status_string(0) == "ok"
    for s in (-1, -2, -3, -4, -99):
        assert isinstance(pb.prism_status_string(s), str) and pb.prism_status_string(s)


def test_workspace_queries(lib):
    p = pb.make_params(32, 8, 131072, 128)
    n = pb.prism_estimate_workspace_bytes(p)
    heads, N = 40, 1024
    assert n >= heads * N * 128 * 2 * 6 + heads * N * 16      # two bands x three bf16 terms
    assert n < 72 << 20
    ws = pb.prism_sparse_attn_workspace_bytes(p)
    # V^T image in bf16 and (whole blocks of 128) in fp16, plus the queue tables
    assert 2 * 8 * 131072 * 128 * 2 + 8 * 1024 * 4 <= ws < 2 * 8 * 131072 * 128 * 2 + (1 << 20)


@pytest.mark.parametrize("kw,status", [
    (dict(n_q_heads=6, n_kv_heads=4), -1),          # h % h_kv
    (dict(n_q_heads=0), -1),
    (dict(head_dim=96), -2),
    (dict(head_dim=512), -2),
    (dict(block=32), -2),
    (dict(seq_len=0), -1),
    (dict(seq_len=128 * 4096), -2),                  # N > 2048
])
def test_bad_geometry_is_rejected(lib, kw, status):
    base = dict(n_q_heads=4, n_kv_heads=2, seq_len=1024, block=128)
    base.update(kw)
    p = pb.make_params(**base)
    n = ctypes.c_size_t(0)
    assert lib.prism_estimate_workspace_bytes(ctypes.byref(p), ctypes.byref(n)) == status
    assert lib.prism_sparse_attn_workspace_bytes(ctypes.byref(p), ctypes.byref(n)) == status


@pytest.mark.parametrize("kw", [dict(d_high=-32), dict(d_low=160), dict(d_high=0, d_low=0),
                                dict(top_p=0.0), dict(top_p=1.5), dict(top_p=float("nan"))])
def test_bad_bands_are_rejected_before_launch(lib, kw):
    base = dict(n_q_heads=4, n_kv_heads=2, seq_len=1024, block=128)
    base.update(kw)
    p = pb.make_params(**base)
    fake = ctypes.c_void_p(256)     # never dereferenced: validation fails first
    rc = lib.prism_estimate(ctypes.byref(p), fake, fake, fake, fake, fake, 10, fake, fake, 1 << 30, None)
    assert rc == -1


@pytest.mark.parametrize("high,low", [
    ([(0, 64), (32, 64)], [(32, 96)]),             # slices of one band overlap
    ([(120, 16)], [(32, 96)]),                     # runs past the head dim
    ([(0, 0)], [(32, 96)]),                        # empty slice
    ([(-8, 16)], [(32, 96)]),
    ([], []),                                      # both bands off
])
def test_bad_band_descriptors_are_rejected_before_launch(lib, high, low):
    p = pb.make_params(4, 2, 1024, 128)
    bands = pb.make_bands(high, low)
    fake = ctypes.c_void_p(256)     # never dereferenced: validation fails first
    rc = lib.prism_estimate_bands(ctypes.byref(p), ctypes.byref(bands), fake, fake, fake, fake, fake, 10,
                                  fake, fake, 1 << 30, None)
    assert rc == -1
    bands.high.n_segments = 9                      # more than PRISM_MAX_SEGMENTS
    assert lib.prism_estimate_bands(ctypes.byref(p), ctypes.byref(bands), fake, fake, fake, fake, fake,
                                    10, fake, fake, 1 << 30, None) == -1
    assert lib.prism_estimate_bands(ctypes.byref(p), None, fake, fake, fake, fake, fake, 10, fake, fake,
                                    1 << 30, None) == -1


def test_bidirectional_capacity_and_pair_limit(lib):
    p = pb.make_params(4, 2, 1024, 128, flags=pb.PRISM_FLAG_BIDIRECTIONAL)
    fake = ctypes.c_void_p(256)
    N = 8
    assert lib.prism_dense_csr(ctypes.byref(p), fake, fake, 4 * N * N - 1, None) == -1   # needs h*N*N
    assert lib.prism_causal_csr(ctypes.byref(p), fake, fake, 4 * N * (N + 1) // 2 - 1, None) == -1
    big = pb.make_params(512, 512, 128 * 2048, 128, flags=pb.PRISM_FLAG_BIDIRECTIONAL)   # h*N*N >= 2^31
    n = ctypes.c_size_t(0)
    assert lib.prism_estimate_workspace_bytes(ctypes.byref(big), ctypes.byref(n)) == -2
    big.flags = 0                                                                          # h*N*(N+1)/2 fits
    assert lib.prism_estimate_workspace_bytes(ctypes.byref(big), ctypes.byref(n)) == 0


def test_null_pointers_and_workspace_are_rejected(lib):
    p = pb.make_params(4, 2, 1024, 128)
    fake = ctypes.c_void_p(256)
    assert lib.prism_estimate(ctypes.byref(p), None, fake, fake, fake, fake, 10, fake, fake, 1 << 30, None) == -1
    assert lib.prism_estimate(ctypes.byref(p), fake, fake, fake, fake, fake, 10, fake, None, 1 << 30, None) == -3
    assert lib.prism_estimate(ctypes.byref(p), fake, fake, fake, fake, fake, 10, fake, fake, 16, None) == -3
    assert lib.prism_estimate(ctypes.byref(p), fake, fake, fake, fake, fake, 10, fake,
                              ctypes.c_void_p(264), 1 << 30, None) == -3           # misaligned
    assert lib.prism_sparse_attn(ctypes.byref(p), fake, fake, None, fake, fake, 0, fake, None, fake, 1 << 30, None) == -1
    assert lib.prism_sparse_attn(ctypes.byref(p), fake, fake, fake, fake, fake, 0, fake, None, fake, 16, None) == -3
    assert lib.prism_causal_csr(ctypes.byref(p), fake, fake, 3, None) == -1        # capacity too small
    assert lib.prism_mask_to_csr(ctypes.byref(p), None, fake, fake, 3, fake, None) == -1
    assert lib.prism_estimate(None, fake, fake, fake, fake, fake, 10, fake, fake, 1 << 30, None) == -1


@pytest.mark.parametrize("kw", [
    dict(base=1.0), dict(base=float("nan")), dict(base=1e4, position_offset=-1),
    dict(base=1e4, position_offset=(1 << 30)),
    dict(base=1e6, yarn_native_len=32768, yarn_scale=0.5),
    dict(base=1e6, yarn_native_len=32768, yarn_scale=4.0, yarn_alpha=32.0, yarn_beta=32.0),
    dict(base=1e6, yarn_native_len=-5, yarn_scale=4.0),
])
def test_bad_rope_descriptors_are_rejected_before_launch(lib, kw):
    p = pb.make_params(4, 2, 1024, 128)
    fake = ctypes.c_void_p(256)
    rope = pb.make_rope(**kw)
    call = lambda r, qi=fake: lib.prism_rope_estimate(ctypes.byref(p), r, None, qi, fake, fake, fake, fake, fake,
                                                      fake, 10, fake, fake, 1 << 30, None)
    assert call(ctypes.byref(rope)) == -1
    assert call(None) == -1                                           # no descriptor at all
    assert call(ctypes.byref(pb.make_rope(1e4)), None) == -1          # null input with a good descriptor


def test_head_dims_64_128_256_are_accepted(lib):
    for d in (64, 128, 256):
        p = pb.make_params(4, 2, 4096, 128, d_high=d // 2, d_low=d // 2, head_dim=d)
        assert pb.prism_estimate_workspace_bytes(p) > 0
        assert pb.prism_sparse_attn_workspace_bytes(p) >= 2 * 4096 * d * 2


def test_varlen_layout_and_malformed_offsets(lib):
    params = pb.make_params(2, 1, 1000, 128)
    mo, ro, co = pb.prism_varlen_layout(params, [0, 300, 1000])
    # N = 3 and 6 blocks: words 2*3*1 and 2*6*1, rows 2*3+1 and 2*6+1, pairs 2*6 and 2*21
    assert mo == [0, 6, 18] and ro == [0, 7, 20] and co == [0, 12, 54]
    for cu in ([0, 500, 400, 1000], [1, 1000], [0, 1001], [0, 500, 500, 1000], [0, 999]):
        with pytest.raises(pb.PrismError):
            pb.prism_varlen_layout(params, cu)
    # a sequence beyond the per-sequence block limit
    big = pb.make_params(1, 1, 64 * 2049 + 64, 64)
    with pytest.raises(pb.PrismError):
        pb.prism_varlen_layout(big, [0, 64 * 2049, 64 * 2049 + 64])
    # a batch longer than one sequence may be is fine
    ok = pb.make_params(1, 1, 2 * 64 * 2048, 64)
    mo, ro, co = pb.prism_varlen_layout(ok, [0, 64 * 2048, 2 * 64 * 2048])
    assert ro == [0, 2049, 4098]
    assert pb.prism_estimate_varlen_workspace_bytes(ok, [0, 64 * 2048, 2 * 64 * 2048]) == \
        pb.prism_estimate_workspace_bytes(pb.make_params(1, 1, 64 * 2048, 64))
    assert pb.prism_sparse_attn_varlen_workspace_bytes(params, [0, 300, 1000]) == \
        pb.prism_sparse_attn_workspace_bytes(pb.make_params(2, 1, 700, 128))


def test_mask_pack_roundtrip():
    import numpy as np
    from tests.gpu_util import pack_mask, unpack_mask
    rng = np.random.default_rng(0)
    for N in (1, 5, 64, 65, 130):
        m = rng.random((3, N, N)) < 0.3
        w = pack_mask(m)
        assert w.shape == (3, N, (N + 63) // 64)
        np.testing.assert_array_equal(unpack_mask(w, N), m)
        assert ((w[0, 0, 0] >> np.uint64(0)) & np.uint64(1)) == m[0, 0, 0]
