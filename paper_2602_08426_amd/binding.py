"""ctypes binding of libprism.so — argument marshalling only.

Every function has the name of the C entry point it calls (include/prism.h).  PyTorch is
used for device memory (`torch.empty`) and the current HIP stream; all computation happens
inside the library's kernels.  There is no fallback: if the library is missing or a call
returns an error status, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

# PRISM_LIBRARY names another build of the same library (the measurement-only variants that
# `python -m paper_2602_08426_amd.build --ablation` writes); there is still no fallback.
_LIB_PATH = os.environ.get("PRISM_LIBRARY") or os.path.join(os.path.dirname(os.path.abspath(__file__)),
                                                            "libprism.so")
_lib: Optional[ctypes.CDLL] = None

PRISM_FLAG_NO_CALIBRATION = 1
PRISM_FLAG_BIDIRECTIONAL = 2
PRISM_FLAG_FORCE_DIAGONAL = 4
PRISM_FLAG_FORCE_SINK = 8
PRISM_FLAG_PAIR_KERNEL = 0x10000000
PRISM_FLAG_GENERAL_KERNEL = 0x20000000
PRISM_FLAG_STREAM_ONLY = 0x40000000
PRISM_MAX_SEGMENTS = 8


class PrismError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _load().prism_status_string(status).decode()
        super().__init__(f"{where} failed with status {status}: {msg}")


class prism_params(ctypes.Structure):
    _fields_ = [("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("seq_len", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("block", ctypes.c_int32), ("d_high", ctypes.c_int32), ("d_low", ctypes.c_int32),
                ("top_p", ctypes.c_float), ("flags", ctypes.c_uint32)]

    @property
    def n_blocks(self) -> int:
        return -(-self.seq_len // self.block)

    @property
    def words_per_row(self) -> int:
        return (self.n_blocks + 63) // 64


class prism_band(ctypes.Structure):
    _fields_ = [("n_segments", ctypes.c_int32), ("start", ctypes.c_int32 * PRISM_MAX_SEGMENTS),
                ("width", ctypes.c_int32 * PRISM_MAX_SEGMENTS)]


class prism_bands(ctypes.Structure):
    _fields_ = [("high", prism_band), ("low", prism_band)]


class prism_rope(ctypes.Structure):
    _fields_ = [("base", ctypes.c_double), ("position_offset", ctypes.c_int32),
                ("yarn_native_len", ctypes.c_int32), ("yarn_scale", ctypes.c_double),
                ("yarn_alpha", ctypes.c_double), ("yarn_beta", ctypes.c_double)]


EXPORTS = ("prism_version", "prism_status_string", "prism_estimate_workspace_bytes",
           "prism_estimate", "prism_estimate_static", "prism_estimate_bands", "prism_rope_estimate", "prism_block_scores",
           "prism_block_scores_bands", "prism_mask_to_csr", "prism_causal_csr", "prism_dense_csr",
           "prism_sparse_attn_workspace_bytes", "prism_sparse_attn", "prism_v_image",
           "prism_sparse_attn_pre", "prism_varlen_layout", "prism_estimate_varlen_workspace_bytes",
           "prism_estimate_varlen", "prism_sparse_attn_varlen_workspace_bytes", "prism_sparse_attn_varlen")


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} not found: build it first (python -m paper_2602_08426_amd.build "
            "or __graft_entry__.build())")
    lib = ctypes.CDLL(_LIB_PATH)
    P, vp, i64, sz = ctypes.POINTER(prism_params), ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t
    PB = ctypes.POINTER(prism_bands)
    lib.prism_version.restype = ctypes.c_int
    lib.prism_version.argtypes = []
    lib.prism_status_string.restype = ctypes.c_char_p
    lib.prism_status_string.argtypes = [ctypes.c_int]
    lib.prism_estimate_workspace_bytes.argtypes = [P, ctypes.POINTER(sz)]
    lib.prism_estimate.argtypes = [P, vp, vp, vp, vp, vp, i64, vp, vp, sz, vp]
    lib.prism_estimate_static.argtypes = [P, vp, vp, vp, vp, vp, i64, vp, vp]
    lib.prism_estimate_bands.argtypes = [P, PB, vp, vp, vp, vp, vp, i64, vp, vp, sz, vp]
    lib.prism_rope_estimate.argtypes = [P, ctypes.POINTER(prism_rope), PB, vp, vp, vp, vp, vp, vp, vp,
                                        i64, vp, vp, sz, vp]
    lib.prism_block_scores.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.prism_block_scores_bands.argtypes = [P, PB, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.prism_dense_csr.argtypes = [P, vp, vp, i64, vp]
    lib.prism_mask_to_csr.argtypes = [P, vp, vp, vp, i64, vp, vp]
    lib.prism_causal_csr.argtypes = [P, vp, vp, i64, vp]
    lib.prism_sparse_attn_workspace_bytes.argtypes = [P, ctypes.POINTER(sz)]
    lib.prism_sparse_attn.argtypes = [P, vp, vp, vp, vp, vp, i64, vp, vp, vp, sz, vp]
    lib.prism_v_image.argtypes = [P, vp, vp, sz, vp]
    lib.prism_sparse_attn_pre.argtypes = [P, vp, vp, vp, sz, vp, vp, i64, vp, vp, vp]
    I32P, I64P = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)
    lib.prism_varlen_layout.argtypes = [P, I32P, ctypes.c_int, I64P, I64P, I64P]
    lib.prism_estimate_varlen_workspace_bytes.argtypes = [P, I32P, ctypes.c_int, ctypes.POINTER(sz)]
    lib.prism_estimate_varlen.argtypes = [P, I32P, ctypes.c_int, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.prism_sparse_attn_varlen_workspace_bytes.argtypes = [P, I32P, ctypes.c_int, ctypes.POINTER(sz)]
    lib.prism_sparse_attn_varlen.argtypes = [P, I32P, ctypes.c_int, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    for name in EXPORTS[2:]:
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def library_path() -> str:
    return _LIB_PATH


def make_params(n_q_heads: int, n_kv_heads: int, seq_len: int, block: int, d_high: int = 64,
                d_low: int = 96, top_p: float = 0.95, flags: int = 0, head_dim: int = 128) -> prism_params:
    return prism_params(n_q_heads, n_kv_heads, seq_len, head_dim, block, d_high, d_low, top_p, flags)


def make_bands(high, low) -> prism_bands:
    """Band descriptors from two lists of (start, width) slices of the head dim."""
    b = prism_bands()
    for band, segs in ((b.high, high), (b.low, low)):
        segs = list(segs)
        if len(segs) > PRISM_MAX_SEGMENTS:
            raise ValueError(f"at most {PRISM_MAX_SEGMENTS} slices per band")
        band.n_segments = len(segs)
        for i, (start, width) in enumerate(segs):
            band.start[i], band.width[i] = start, width
    return b


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(status: int, where: str) -> None:
    if status != 0:
        raise PrismError(status, where)


def prism_version() -> int:
    return _load().prism_version()


def prism_status_string(status: int) -> str:
    return _load().prism_status_string(status).decode()


def prism_estimate_workspace_bytes(params: prism_params) -> int:
    n = ctypes.c_size_t(0)
    _check(_load().prism_estimate_workspace_bytes(ctypes.byref(params), ctypes.byref(n)),
           "prism_estimate_workspace_bytes")
    return n.value


def prism_sparse_attn_workspace_bytes(params: prism_params) -> int:
    n = ctypes.c_size_t(0)
    _check(_load().prism_sparse_attn_workspace_bytes(ctypes.byref(params), ctypes.byref(n)),
           "prism_sparse_attn_workspace_bytes")
    return n.value


def alloc_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    """256-byte aligned scratch (torch's caching allocator aligns to 512 B)."""
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def alloc_estimate_outputs(params: prism_params, col_capacity: Optional[int] = None, device="cuda"):
    N, W, h = params.n_blocks, params.words_per_row, params.n_q_heads
    if col_capacity is None:
        col_capacity = h * N * N if params.flags & PRISM_FLAG_BIDIRECTIONAL else h * N * (N + 1) // 2
    mask_bits = torch.empty((h, N, W), dtype=torch.int64, device=device)
    row_ptr = torch.empty(h * N + 1, dtype=torch.int32, device=device)
    col_idx = torch.empty(max(col_capacity, 1), dtype=torch.int32, device=device)
    info = torch.empty(4, dtype=torch.int32, device=device)
    return mask_bits, row_ptr, col_idx, info


def prism_estimate(params: prism_params, q: torch.Tensor, k: torch.Tensor, mask_bits: torch.Tensor,
                   row_ptr: torch.Tensor, col_idx: torch.Tensor, col_capacity: int,
                   info: torch.Tensor, workspace: torch.Tensor) -> None:
    _check(_load().prism_estimate(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(mask_bits),
                                  _ptr(row_ptr), _ptr(col_idx), col_capacity, _ptr(info),
                                  _ptr(workspace), workspace.numel(), _stream()), "prism_estimate")


def prism_estimate_static(params: prism_params, q: torch.Tensor, k: torch.Tensor,
                          mask_bits: torch.Tensor, row_ptr: torch.Tensor, col_idx: torch.Tensor,
                          col_capacity: int, info: torch.Tensor) -> None:
    _check(_load().prism_estimate_static(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(mask_bits),
                                         _ptr(row_ptr), _ptr(col_idx), col_capacity, _ptr(info),
                                         _stream()), "prism_estimate_static")


def prism_estimate_bands(params: prism_params, bands: prism_bands, q: torch.Tensor, k: torch.Tensor,
                         mask_bits: torch.Tensor, row_ptr: torch.Tensor, col_idx: torch.Tensor,
                         col_capacity: int, info: torch.Tensor, workspace: torch.Tensor) -> None:
    _check(_load().prism_estimate_bands(ctypes.byref(params), ctypes.byref(bands), _ptr(q), _ptr(k),
                                        _ptr(mask_bits), _ptr(row_ptr), _ptr(col_idx), col_capacity,
                                        _ptr(info), _ptr(workspace), workspace.numel(), _stream()),
           "prism_estimate_bands")


def make_rope(base: float, position_offset: int = 0, yarn_native_len: int = 0, yarn_scale: float = 1.0,
              yarn_alpha: float = 1.0, yarn_beta: float = 32.0) -> prism_rope:
    return prism_rope(base, position_offset, yarn_native_len, yarn_scale, yarn_alpha, yarn_beta)


def prism_rope_estimate(params: prism_params, rope: prism_rope, bands: Optional[prism_bands],
                        q_in: torch.Tensor, k_in: torch.Tensor, q_out: torch.Tensor, k_out: torch.Tensor,
                        mask_bits: torch.Tensor, row_ptr: torch.Tensor, col_idx: torch.Tensor,
                        col_capacity: int, info: torch.Tensor, workspace: torch.Tensor) -> None:
    _check(_load().prism_rope_estimate(ctypes.byref(params), ctypes.byref(rope),
                                       ctypes.byref(bands) if bands is not None else None,
                                       _ptr(q_in), _ptr(k_in), _ptr(q_out), _ptr(k_out), _ptr(mask_bits),
                                       _ptr(row_ptr), _ptr(col_idx), col_capacity, _ptr(info),
                                       _ptr(workspace), workspace.numel(), _stream()),
           "prism_rope_estimate")


def prism_block_scores(params: prism_params, q: torch.Tensor, k: torch.Tensor,
                       pooled_q: Optional[torch.Tensor], pooled_k: Optional[torch.Tensor],
                       scales: Optional[torch.Tensor], logits_high: Optional[torch.Tensor],
                       logits_low: Optional[torch.Tensor], workspace: torch.Tensor) -> None:
    _check(_load().prism_block_scores(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(pooled_q),
                                      _ptr(pooled_k), _ptr(scales), _ptr(logits_high),
                                      _ptr(logits_low), _ptr(workspace), workspace.numel(),
                                      _stream()), "prism_block_scores")


def prism_block_scores_bands(params: prism_params, bands: prism_bands, q: torch.Tensor,
                             k: torch.Tensor, pooled_q: Optional[torch.Tensor],
                             pooled_k: Optional[torch.Tensor], scales: Optional[torch.Tensor],
                             logits_high: Optional[torch.Tensor], logits_low: Optional[torch.Tensor],
                             workspace: torch.Tensor) -> None:
    _check(_load().prism_block_scores_bands(ctypes.byref(params), ctypes.byref(bands), _ptr(q),
                                            _ptr(k), _ptr(pooled_q), _ptr(pooled_k), _ptr(scales),
                                            _ptr(logits_high), _ptr(logits_low), _ptr(workspace),
                                            workspace.numel(), _stream()), "prism_block_scores_bands")


def prism_mask_to_csr(params: prism_params, mask_bits: torch.Tensor, row_ptr: torch.Tensor,
                      col_idx: torch.Tensor, col_capacity: int, info: torch.Tensor) -> None:
    _check(_load().prism_mask_to_csr(ctypes.byref(params), _ptr(mask_bits), _ptr(row_ptr),
                                     _ptr(col_idx), col_capacity, _ptr(info), _stream()),
           "prism_mask_to_csr")


def prism_causal_csr(params: prism_params, row_ptr: torch.Tensor, col_idx: torch.Tensor,
                     col_capacity: int) -> None:
    _check(_load().prism_causal_csr(ctypes.byref(params), _ptr(row_ptr), _ptr(col_idx),
                                    col_capacity, _stream()), "prism_causal_csr")


def prism_dense_csr(params: prism_params, row_ptr: torch.Tensor, col_idx: torch.Tensor,
                    col_capacity: int) -> None:
    _check(_load().prism_dense_csr(ctypes.byref(params), _ptr(row_ptr), _ptr(col_idx),
                                   col_capacity, _stream()), "prism_dense_csr")


def prism_sparse_attn(params: prism_params, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                      row_ptr: torch.Tensor, col_idx: torch.Tensor, col_count: int,
                      out: torch.Tensor, lse: Optional[torch.Tensor], workspace: torch.Tensor) -> None:
    _check(_load().prism_sparse_attn(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(v), _ptr(row_ptr),
                                     _ptr(col_idx), col_count, _ptr(out), _ptr(lse),
                                     _ptr(workspace), workspace.numel(), _stream()),
           "prism_sparse_attn")


def prism_v_image(params: prism_params, v: torch.Tensor, v_image: torch.Tensor) -> None:
    _check(_load().prism_v_image(ctypes.byref(params), _ptr(v), _ptr(v_image), v_image.numel(),
                                 _stream()), "prism_v_image")


def prism_sparse_attn_pre(params: prism_params, q: torch.Tensor, k: torch.Tensor,
                          v_image: torch.Tensor, row_ptr: torch.Tensor, col_idx: torch.Tensor,
                          col_count: int, out: torch.Tensor, lse: Optional[torch.Tensor]) -> None:
    _check(_load().prism_sparse_attn_pre(ctypes.byref(params), _ptr(q), _ptr(k), _ptr(v_image),
                                         v_image.numel(), _ptr(row_ptr), _ptr(col_idx), col_count,
                                         _ptr(out), _ptr(lse), _stream()), "prism_sparse_attn_pre")


# ---- packed variable-length batches ---------------------------------------------------------
def _cu(cu_seqlens):
    """host int32 array of sequence offsets -> (ctypes array, number of sequences)"""
    vals = [int(x) for x in cu_seqlens]
    return (ctypes.c_int32 * len(vals))(*vals), len(vals) - 1


def prism_varlen_layout(params: prism_params, cu_seqlens):
    """(mask_offsets, row_offsets, col_offsets): lists of n_seqs + 1 ints, last = total."""
    cu, n = _cu(cu_seqlens)
    outs = [(ctypes.c_int64 * (n + 1))() for _ in range(3)]
    _check(_load().prism_varlen_layout(ctypes.byref(params), cu, n, *outs), "prism_varlen_layout")
    return tuple(list(o) for o in outs)


def prism_estimate_varlen_workspace_bytes(params: prism_params, cu_seqlens) -> int:
    cu, n = _cu(cu_seqlens)
    nb = ctypes.c_size_t(0)
    _check(_load().prism_estimate_varlen_workspace_bytes(ctypes.byref(params), cu, n, ctypes.byref(nb)),
           "prism_estimate_varlen_workspace_bytes")
    return nb.value


def prism_estimate_varlen(params: prism_params, cu_seqlens, q: torch.Tensor, k: torch.Tensor,
                          mask_bits: torch.Tensor, row_ptr: torch.Tensor, col_idx: torch.Tensor,
                          info: torch.Tensor, workspace: torch.Tensor) -> None:
    cu, n = _cu(cu_seqlens)
    _check(_load().prism_estimate_varlen(ctypes.byref(params), cu, n, _ptr(q), _ptr(k), _ptr(mask_bits),
                                         _ptr(row_ptr), _ptr(col_idx), _ptr(info), _ptr(workspace),
                                         workspace.numel(), _stream()), "prism_estimate_varlen")


def prism_sparse_attn_varlen_workspace_bytes(params: prism_params, cu_seqlens) -> int:
    cu, n = _cu(cu_seqlens)
    nb = ctypes.c_size_t(0)
    _check(_load().prism_sparse_attn_varlen_workspace_bytes(ctypes.byref(params), cu, n, ctypes.byref(nb)),
           "prism_sparse_attn_varlen_workspace_bytes")
    return nb.value


def prism_sparse_attn_varlen(params: prism_params, cu_seqlens, q: torch.Tensor, k: torch.Tensor,
                             v: torch.Tensor, row_ptr: torch.Tensor, col_idx: torch.Tensor,
                             out: torch.Tensor, lse: Optional[torch.Tensor], workspace: torch.Tensor) -> None:
    cu, n = _cu(cu_seqlens)
    _check(_load().prism_sparse_attn_varlen(ctypes.byref(params), cu, n, _ptr(q), _ptr(k), _ptr(v),
                                            _ptr(row_ptr), _ptr(col_idx), _ptr(out), _ptr(lse),
                                            _ptr(workspace), workspace.numel(), _stream()),
           "prism_sparse_attn_varlen")


# ---- conveniences for callers holding numpy bf16 bit patterns --------------------------
def bf16_bits_to_device(bits, device="cuda") -> torch.Tensor:
    """numpy uint16 bf16 bit patterns -> device bf16 tensor (a copy, no arithmetic)."""
    import numpy as np
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.to(device).view(torch.bfloat16)


def device_bf16_to_bits(t: torch.Tensor):
    """device bf16 tensor -> numpy uint16 bit patterns."""
    import numpy as np
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
