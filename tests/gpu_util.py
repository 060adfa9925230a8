"""Helpers shared by the GPU parity tests: move seeded inputs to the device, call the C ABI
through the binding, bring results back as numpy."""
from __future__ import annotations

import numpy as np
import torch

from paper_2602_08426_amd import binding as pb


def unpack_mask(mask_words: np.ndarray, N: int) -> np.ndarray:
    """[h, N, W] uint64 words -> [h, N, N] bool."""
    h, _, W = mask_words.shape
    bits = np.unpackbits(mask_words.view(np.uint8).reshape(h, N, W * 8), axis=-1, bitorder="little")
    return bits[:, :, :N].astype(bool)


def pack_mask(mask: np.ndarray) -> np.ndarray:
    """[h, N, N] bool -> [h, N, W] uint64 words (bit v%64 of word v//64)."""
    h, N, _ = mask.shape
    W = (N + 63) // 64
    padded = np.zeros((h, N, W * 64), dtype=np.uint8)
    padded[:, :, :N] = mask
    return np.packbits(padded, axis=-1, bitorder="little").view(np.uint64).reshape(h, N, W)


def params_for(w, **over):
    kw = dict(n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, seq_len=w.seq_len, block=w.block,
              d_high=w.d_high, d_low=w.d_low, top_p=w.top_p, head_dim=w.head_dim)
    kw.update(over)
    return pb.make_params(**kw)


def gpu_estimate(params, q_dev, k_dev, col_capacity=None, bands=None):
    """Returns dict of numpy results of prism_estimate (prism_estimate_bands with `bands`)."""
    mask_bits, row_ptr, col_idx, info = pb.alloc_estimate_outputs(params, col_capacity)
    cap = col_idx.numel() if col_capacity is None else col_capacity
    ws = pb.alloc_workspace(pb.prism_estimate_workspace_bytes(params))
    if bands is None:
        pb.prism_estimate(params, q_dev, k_dev, mask_bits, row_ptr, col_idx, cap, info, ws)
    else:
        pb.prism_estimate_bands(params, bands, q_dev, k_dev, mask_bits, row_ptr, col_idx, cap, info, ws)
    torch.cuda.synchronize()
    N = params.n_blocks
    words = mask_bits.cpu().numpy().view(np.uint64)
    return dict(mask=unpack_mask(words, N), words=words, row_ptr=row_ptr.cpu().numpy(),
                col_idx=col_idx.cpu().numpy(), info=info.cpu().numpy(),
                dev=(mask_bits, row_ptr, col_idx, info))


def gpu_block_scores(params, q_dev, k_dev, want_logits=True, bands=None):
    h, hk, N, d = params.n_q_heads, params.n_kv_heads, params.n_blocks, params.head_dim
    pq = torch.empty((h, N, d), dtype=torch.float32, device="cuda")
    pk = torch.empty((hk, N, d), dtype=torch.float32, device="cuda")
    sc = torch.empty((h, 2), dtype=torch.float32, device="cuda")
    lh = torch.full((h, N, N), float("nan"), dtype=torch.float32, device="cuda") if want_logits else None
    ll = torch.full((h, N, N), float("nan"), dtype=torch.float32, device="cuda") if want_logits else None
    ws = pb.alloc_workspace(pb.prism_estimate_workspace_bytes(params))
    if bands is None:
        pb.prism_block_scores(params, q_dev, k_dev, pq, pk, sc, lh, ll, ws)
    else:
        pb.prism_block_scores_bands(params, bands, q_dev, k_dev, pq, pk, sc, lh, ll, ws)
    torch.cuda.synchronize()
    out = dict(pooled_q=pq.cpu().numpy(), pooled_k=pk.cpu().numpy(), scales=sc.cpu().numpy())
    if want_logits:
        out["logits_high"] = lh.cpu().numpy()
        out["logits_low"] = ll.cpu().numpy()
    return out


def gpu_sparse_attn(params, q_dev, k_dev, v_dev, row_ptr_dev, col_idx_dev, col_count, want_lse=True):
    h, L = params.n_q_heads, params.seq_len
    out = torch.full((h, L, params.head_dim), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((h, L), float("nan"), dtype=torch.float32, device="cuda") if want_lse else None
    ws = pb.alloc_workspace(pb.prism_sparse_attn_workspace_bytes(params))
    pb.prism_sparse_attn(params, q_dev, k_dev, v_dev, row_ptr_dev, col_idx_dev, col_count, out, lse, ws)
    torch.cuda.synchronize()
    return out, lse


def csr_to_device(row_ptr: np.ndarray, col_idx: np.ndarray):
    rp = torch.from_numpy(row_ptr.astype(np.int32)).cuda()
    ci = torch.from_numpy(np.concatenate([col_idx.astype(np.int32), np.zeros(1, np.int32)])).cuda()
    return rp, ci, int(len(col_idx))


def bf16_out_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy().astype(np.float64)
