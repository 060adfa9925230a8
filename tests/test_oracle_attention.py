"""Pins for the attention half of the CPU oracle (no GPU): naive scalar loops on tiny
sizes, a library routine (torch SDPA in fp64) for dense causal attention, and the
special cases all-ones mask == dense and diagonal-only mask == per-block attention."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import prism_oracle as orc


def _naive(Q, K, V, mask, B, causal=True):
    """Token-by-token definition with Python scalars: softmax over visible keys."""
    h, L, d = Q.shape
    g = h // K.shape[0]
    O = np.zeros((h, L, d))
    lse = np.full((h, L), -math.inf)
    for hq in range(h):
        kv = hq // g
        for i in range(L):
            vis = [j for j in range(i + 1 if causal else L) if mask[hq, i // B, j // B]]
            if not vis:
                continue
            s = [sum(Q[hq, i, c] * K[kv, j, c] for c in range(d)) / math.sqrt(d) for j in vis]
            mx = max(s)
            e = [math.exp(x - mx) for x in s]
            den = sum(e)
            for c in range(d):
                O[hq, i, c] = sum(e[t] * V[kv, j, c] for t, j in enumerate(vis)) / den
            lse[hq, i] = mx + math.log(den)
    return O, lse


@pytest.mark.parametrize("seed,h,h_kv,L,B,d", [(0, 2, 1, 24, 4, 4), (1, 4, 2, 20, 4, 8), (2, 1, 1, 21, 8, 4)])
def test_block_sparse_matches_naive_loops(seed, h, h_kv, L, B, d):
    rng = np.random.default_rng(seed)
    Q = rng.standard_normal((h, L, d)); K = rng.standard_normal((h_kv, L, d)); V = rng.standard_normal((h_kv, L, d))
    N = -(-L // B)
    mask = np.tril(rng.random((h, N, N)) < 0.5)
    mask[:, 2, :] = False                                  # one empty row per head
    ref_o, ref_l = _naive(Q, K, V, mask, B)
    got = orc.block_sparse_attention(Q, K, V, mask, B)
    for (hq, u), (o, l) in got.items():
        r0, r1 = u * B, min(L, (u + 1) * B)
        np.testing.assert_allclose(o, ref_o[hq, r0:r1], atol=1e-13)
        np.testing.assert_allclose(l, ref_l[hq, r0:r1], atol=1e-13)


def test_bidirectional_block_sparse_matches_naive_loops_and_sdpa():
    """causal=False: every token of a listed block is visible; the all-ones mask is plain
    softmax attention (checked against torch SDPA in fp64)."""
    rng = np.random.default_rng(7)
    h, h_kv, L, B, d = 4, 2, 24, 4, 8
    Q = rng.standard_normal((h, L, d)); K = rng.standard_normal((h_kv, L, d)); V = rng.standard_normal((h_kv, L, d))
    N = L // B
    mask = rng.random((h, N, N)) < 0.5
    mask[:, 1, :] = False
    ref_o, ref_l = _naive(Q, K, V, mask, B, causal=False)
    got = orc.block_sparse_attention(Q, K, V, mask, B, causal=False)
    for (hq, u), (o, l) in got.items():
        np.testing.assert_allclose(o, ref_o[hq, u * B:(u + 1) * B], atol=1e-13)
        np.testing.assert_allclose(l, ref_l[hq, u * B:(u + 1) * B], atol=1e-13)
    assert (mask & ~np.tril(np.ones((N, N), bool))).any()          # blocks above the diagonal were used
    full_o, full_l = orc.dense_full_attention(Q, K, V)
    ones = np.ones((h, N, N), bool)
    for (hq, u), (o, l) in orc.block_sparse_attention(Q, K, V, ones, B, causal=False).items():
        np.testing.assert_allclose(o, full_o[hq, u * B:(u + 1) * B], atol=1e-13)
        np.testing.assert_allclose(l, full_l[hq, u * B:(u + 1) * B], atol=1e-13)
    tq, tk, tv = (torch.from_numpy(x) for x in (Q, K, V))
    ref = F.scaled_dot_product_attention(tq[None], tk.repeat_interleave(h // h_kv, 0)[None],
                                         tv.repeat_interleave(h // h_kv, 0)[None], is_causal=False)[0]
    np.testing.assert_allclose(full_o, ref.numpy(), atol=1e-12)


def test_all_ones_mask_equals_dense():
    rng = np.random.default_rng(3)
    h, h_kv, L, B, d = 4, 2, 96, 16, 16
    Q = rng.standard_normal((h, L, d)); K = rng.standard_normal((h_kv, L, d)); V = rng.standard_normal((h_kv, L, d))
    N = L // B
    ones = np.tril(np.ones((N, N), bool))[None].repeat(h, 0)
    sp = orc.block_sparse_attention(Q, K, V, ones, B)
    dn_o, dn_l = orc.dense_causal_attention(Q, K, V, q_chunk=40)
    for (hq, u), (o, l) in sp.items():
        np.testing.assert_allclose(o, dn_o[hq, u * B:(u + 1) * B], atol=1e-13)
        np.testing.assert_allclose(l, dn_l[hq, u * B:(u + 1) * B], atol=1e-13)


def test_dense_matches_torch_sdpa_fp64():
    rng = np.random.default_rng(4)
    h, h_kv, L, d = 6, 2, 200, 32
    Q = rng.standard_normal((h, L, d)); K = rng.standard_normal((h_kv, L, d)); V = rng.standard_normal((h_kv, L, d))
    o, lse = orc.dense_causal_attention(Q, K, V, q_chunk=64)
    tq = torch.from_numpy(Q)[None]
    tk = torch.from_numpy(K).repeat_interleave(h // h_kv, 0)[None]
    tv = torch.from_numpy(V).repeat_interleave(h // h_kv, 0)[None]
    ref = F.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].numpy()
    np.testing.assert_allclose(o, ref, atol=1e-12)
    s = (tq[0] @ tk[0].transpose(1, 2)) / math.sqrt(d)
    s = s.masked_fill(~torch.tril(torch.ones(L, L, dtype=torch.bool)), float("-inf"))
    np.testing.assert_allclose(lse, torch.logsumexp(s, -1).numpy(), atol=1e-12)


def test_diagonal_only_mask_is_local_block_attention():
    rng = np.random.default_rng(5)
    h, L, B, d = 2, 64, 16, 8
    Q = rng.standard_normal((h, L, d)); K = rng.standard_normal((h, L, d)); V = rng.standard_normal((h, L, d))
    N = L // B
    diag = np.eye(N, dtype=bool)[None].repeat(h, 0)
    got = orc.block_sparse_attention(Q, K, V, diag, B)
    for (hq, u), (o, _) in got.items():
        sl = slice(u * B, (u + 1) * B)
        ref = F.scaled_dot_product_attention(torch.from_numpy(Q[hq, sl])[None, None],
                                             torch.from_numpy(K[hq, sl])[None, None],
                                             torch.from_numpy(V[hq, sl])[None, None],
                                             is_causal=True)[0, 0].numpy()
        np.testing.assert_allclose(o, ref, atol=1e-13)


def test_softmax_weights_sum_to_one_via_lse():
    rng = np.random.default_rng(6)
    L, B, d = 48, 8, 8
    Q = rng.standard_normal((1, L, d)); K = rng.standard_normal((1, L, d)); V = np.ones((1, L, d))
    N = L // B
    mask = np.tril(rng.random((1, N, N)) < 0.6); mask[0, np.arange(N), np.arange(N)] = True
    got = orc.block_sparse_attention(Q, K, V, mask, B)
    for (hq, u), (o, lse) in got.items():
        np.testing.assert_allclose(o, 1.0, atol=1e-13)      # convex combination of ones
        for r in range(B):
            i = u * B + r
            vis = [j for j in range(i + 1) if mask[0, u, j // B]]
            w = np.exp(Q[0, i] @ K[0, vis].T / math.sqrt(d) - lse[r])
            assert abs(w.sum() - 1.0) < 1e-12


def test_bf16_decode_is_exact():
    bits = np.array([0x3F80, 0xBF80, 0x4049, 0x0000, 0x8000, 0x7F7F, 0x0001], dtype=np.uint16)
    ref = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(orc.bf16_to_f64(bits), ref)
