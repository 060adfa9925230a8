"""CPU oracle for the Prism hot path — TEST INFRASTRUCTURE, not a product path.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this module.  It shares no code with the HIP library or its Python binding and
imports neither; it is a plain, slow, fp64 NumPy statement of what the paper
defines, written to be checked against the paper by eye.

Two parts of different kinds:

* Block selection (heuristic; the algorithm is its own definition): follows the
  steps and notation of the paper's Sec. 3.4 "Prism: Spectral-Aware Block
  Selection" (Fig. "PyTorch-style implementation of Prism") and App. C
  "Top-P Block Selection":
    pool -> band slices -> RMS -> temperatures -> dual-band logits ->
    row softmax -> top-p -> union.
* Block-masked causal attention (exact; has a plain definition): softmax over the
  keys that are both causally visible and inside a selected block
  (Sec. 2 "Block-Sparse Attention", Sec. 3.1 "Coarse-grained Attention" for the
  1/sqrt(d) scale), and dense causal attention as the all-ones special case,
  written as a separate function.

Readings taken where the paper is silent (all listed in the design notes):
  - bands are contiguous slices [0, d_h) and [d - d_l, d) of the adjacent-pair
    RoPE layout; rms() is one scalar per head over all N blocks and the band's
    dims; for grouped-query attention the key statistics are per kv head and
    q-head hq uses kv-head hq // (h / h_kv);
  - estimation is block-causal: logits of key blocks v > u are -inf before the
    softmax; nothing (diagonal, sink) is forced;
  - top-p ties: stable descending order (lower block index first);
  - a band with d_z = 0 is skipped; zero band energy gives zero logits;
  - p >= 1 selects every causal block;
  - a band may be given as a list of (start, width) slices of the head dimension
    instead of one contiguous slice: the band vector is their concatenation and
    d_z the total width.  This covers the axis-wise bands of App. "HunyuanVideo
    Spectral Configuration" (first d_high^a / last d_low^a dims of each axis subspace)
    and RoPE stored as (j, j + d/2) pairs;
  - causal=False (bidirectional attention, the video setting) drops the block-causal
    restriction in the selection and the token-causal one in the attention;
  - force_diagonal / force_sink are optional extras (not in the paper): after the
    union, block u (resp. block 0) of every row is switched on.

rope_frequencies / apply_rope restate Sec. 3.1 and the YaRN appendix; they are pinned by
the zone boundaries the appendix prints, rotation invariants and the Dirichlet closed form.

Pins (tests/test_oracle_*.py): Dirichlet-kernel closed form for pooled RoPE
content (Eq. "attenuation"), printed cutoff dimensions, 1/sqrt(B) residual,
tau = 1 when a band is the full head, brute-force top-p on tiny rows, naive
triple-loop attention, all-ones mask == dense, torch SDPA in fp64.
Exact mask values on random data are pinned by no printed example in the paper
("parity unpinned" for the selection on random data beyond those invariants).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np


# --------------------------------------------------------------------------- #
# input decoding
# --------------------------------------------------------------------------- #
def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact value of bf16 bit patterns (uint16) as fp64."""
    b = np.ascontiguousarray(bits)
    if b.dtype != np.uint16:
        raise TypeError("expected uint16 bf16 bit patterns")
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round finite fp64 values to bf16 (round to nearest, ties to even) and return the bit
    patterns.  Done directly on the fp64 value: the upper 16 bits of the fp32 pattern of the
    nearest bf16, found by comparing with the two neighbouring bf16 values."""
    x = np.asarray(x, dtype=np.float64)
    f = x.astype(np.float32)                                    # only used to locate a neighbour
    lo_bits = f.view(np.uint32) & np.uint32(0xFFFF0000)         # truncation toward zero
    lo = lo_bits.view(np.float32).astype(np.float64)
    # fp32 rounding may have crossed a bf16 boundary away from zero; step back if so
    over = np.abs(lo) > np.abs(x)
    lo_bits = np.where(over, lo_bits - np.uint32(0x10000), lo_bits).astype(np.uint32)
    lo = lo_bits.view(np.float32).astype(np.float64)
    hi_bits = (lo_bits + np.uint32(0x10000)).astype(np.uint32)
    hi = hi_bits.view(np.float32).astype(np.float64)
    d_lo, d_hi = np.abs(x - lo), np.abs(hi - x)
    even_lo = ((lo_bits >> np.uint32(16)) & np.uint32(1)) == 0
    take_hi = (d_hi < d_lo) | ((d_hi == d_lo) & ~even_lo)
    return (np.where(take_hi, hi_bits, lo_bits) >> np.uint32(16)).astype(np.uint16)


# --------------------------------------------------------------------------- #
# Rotary position embedding (Sec. 3.1 "Spectral Structure of RoPE") and the YaRN
# frequency map (App. "Compatibility with YaRN") — used to check the library's fused
# RoPE + pooling producer
# --------------------------------------------------------------------------- #
def rope_frequencies(d: int, base: float,
                     yarn: Optional[Tuple[int, float, float, float]] = None) -> np.ndarray:
    """theta_j = base^(-2j/d) for feature pair j = 0 .. d/2-1 (Sec. 3.1).  With
    yarn = (L, s, alpha, beta): theta'_j = (1 - gamma_j) theta_j / s + gamma_j theta_j where
    gamma_j is 1 for r_j > beta, 0 for r_j < alpha and (r_j - alpha) / (beta - alpha) between,
    r_j = L theta_j / (2 pi) (App. "Compatibility with YaRN", NTK-by-parts interpolation)."""
    j = np.arange(d // 2, dtype=np.float64)
    theta = np.power(float(base), -2.0 * j / d)
    if yarn is None:
        return theta
    L, s, alpha, beta = yarn
    r = L * theta / (2.0 * np.pi)
    gamma = np.where(r > beta, 1.0, np.where(r < alpha, 0.0, (r - alpha) / (beta - alpha)))
    return (1.0 - gamma) * theta / s + gamma * theta


def apply_rope(X: np.ndarray, theta: np.ndarray, position_offset: int = 0) -> np.ndarray:
    """X [..., L, d] -> rotated copy: feature pair j = dims (2j, 2j+1) of the token at position
    n = position_offset + (index along L), read as the complex number x + i y, is multiplied by
    exp(i n theta_j) (Sec. 3.1: x_n^(j) = x_nope^(j) e^{i n theta_j})."""
    X = np.asarray(X, dtype=np.float64)
    L, d = X.shape[-2], X.shape[-1]
    n = position_offset + np.arange(L, dtype=np.float64)
    z = X[..., 0::2] + 1j * X[..., 1::2]
    z = z * np.exp(1j * n[:, None] * np.asarray(theta, dtype=np.float64)[None, :])
    out = np.empty_like(X)
    out[..., 0::2] = z.real
    out[..., 1::2] = z.imag
    return out


# --------------------------------------------------------------------------- #
# Part 1 — block selection, step by step (Sec. 3.4, App. C)
# --------------------------------------------------------------------------- #
def pool(X: np.ndarray, B: int) -> np.ndarray:
    """Mean pooling, Eq. "mean-pooling": x_bar_u = (1/|I_u|) sum_{i in I_u} x_i.

    X: [H, L, d] fp64 -> [H, N, d], N = ceil(L / B).  A ragged last block is
    averaged over the tokens it actually holds."""
    H, L, d = X.shape
    N = -(-L // B)
    out = np.empty((H, N, d), dtype=np.float64)
    for u in range(N):
        out[:, u, :] = X[:, u * B:min(L, (u + 1) * B), :].mean(axis=1)
    return out


def rms(Xb: np.ndarray) -> np.ndarray:
    """RMS(X_bar) = sqrt( (1/N) sum_u ||x_bar_u||^2 / width ), one scalar per head
    (Sec. 3.4 "Energy-Based Temperature Calibration").  Xb: [H, N, width]."""
    H, N, width = Xb.shape
    return np.sqrt((Xb ** 2).sum(axis=(1, 2)) / (N * width))


def temperature(d_z: int, d: int, rq_z: np.ndarray, rq: np.ndarray,
                rk_z: np.ndarray, rk: np.ndarray) -> np.ndarray:
    """tau_z = sqrt(d_z/d) * (RMS(Qbar_z)/RMS(Qbar)) * (RMS(Kbar_z)/RMS(Kbar))."""
    with np.errstate(divide="ignore", invalid="ignore"):
        t = np.sqrt(d_z / d) * (rq_z / rq) * (rk_z / rk)
    return t


def softmax_rows(logits: np.ndarray) -> np.ndarray:
    """Row softmax over the last axis; -inf entries get probability 0."""
    m = logits.max(axis=-1, keepdims=True)
    e = np.exp(logits - m)
    return e / e.sum(axis=-1, keepdims=True)


def top_p(probs: np.ndarray, p: float) -> np.ndarray:
    """Top-p selection of App. C in words: per row, walk the blocks from the most to the
    least probable (equal probabilities: lower index first) and take a block as long as the
    mass of the blocks already taken is below p; the walk stops with the block that carries
    the taken mass to p or beyond, so the result is the smallest set of most probable blocks
    whose mass reaches p.  probs: [..., N] -> bool [..., N]."""
    n = probs.shape[-1]
    rows = np.ascontiguousarray(probs, dtype=np.float64).reshape(-1, n)
    taken = np.zeros(rows.shape, dtype=bool)
    for r in range(rows.shape[0]):
        ranked = np.argsort(-rows[r], kind="stable")
        mass_after = np.add.accumulate(rows[r][ranked])      # mass once rank k has been taken
        reached = np.nonzero(mass_after >= p)[0]
        n_taken = int(reached[0]) + 1 if len(reached) else n
        taken[r, ranked[:n_taken]] = True
    return taken.reshape(probs.shape)


Segments = Sequence[Tuple[int, int]]          # (start, width) slices of the head dim


def band_dims(d: int, d_h: int, d_l: int,
              bands: Optional[Dict[str, Segments]] = None) -> Dict[str, np.ndarray]:
    """Feature dims of the two bands, in band order.  Default (Sec. 3.4, Fig.
    "PyTorch-style implementation"): high = first d_h dims, low = last d_l dims.
    With `bands`, each band is the concatenation of its (start, width) slices."""
    if bands is None:
        bands = {"high": [(0, d_h)] if d_h > 0 else [],
                 "low": [(d - d_l, d_l)] if d_l > 0 else []}
    out = {}
    for z in ("high", "low"):
        idx: List[int] = []
        for start, width in bands.get(z, []):
            if width <= 0 or start < 0 or start + width > d:
                raise ValueError(f"bad segment ({start}, {width}) for head_dim {d}")
            idx.extend(range(start, start + width))
        if len(set(idx)) != len(idx):
            raise ValueError("segments of one band overlap")
        out[z] = np.asarray(idx, dtype=np.int64)
    return out


@dataclass
class Selection:
    """Everything the selection produces for one call (all q-heads)."""
    mask: np.ndarray                 # [h, N, N] bool, union of the bands
    band_masks: Dict[str, np.ndarray]   # "high"/"low" -> [h, N, N] bool
    logits: Dict[str, np.ndarray]    # "high"/"low" -> [h, N, N] fp64 (-inf above diagonal)
    probs: Dict[str, np.ndarray]
    tau: Dict[str, np.ndarray]       # [h]
    scale: Dict[str, np.ndarray]     # sqrt(d_z) * tau_z, [h]
    q_pooled: np.ndarray             # [h, N, d]
    k_pooled: np.ndarray             # [h_kv, N, d]
    rms_q: Dict[str, np.ndarray]     # "full"/"high"/"low" -> [h]
    rms_k: Dict[str, np.ndarray]     # -> [h_kv]
    valid: np.ndarray                # [N, N] bool: block pairs that may be selected at all
    forced: np.ndarray               # [h, N, N] bool: blocks switched on by force_* options


def prism_select(Q: np.ndarray, K: np.ndarray, d_h: int, d_l: int, B: int, p: float,
                 causal: bool = True, calibrate: bool = True,
                 bands: Optional[Dict[str, Segments]] = None,
                 force_diagonal: bool = False, force_sink: bool = False) -> Selection:
    """Block mask of Sec. 3.4.  Q: [h, L, d] fp64, K: [h_kv, L, d] fp64.
    d_h / d_l are ignored when `bands` is given."""
    h, L, d = Q.shape
    h_kv = K.shape[0]
    if h % h_kv:
        raise ValueError("n_q_heads must be a multiple of n_kv_heads")
    kv_of = np.arange(h) // (h // h_kv)            # q-head -> its kv head

    Qb, Kb = pool(Q, B), pool(K, B)                # block means, Eq. "mean-pooling"
    N = Qb.shape[1]
    dims = band_dims(d, d_h, d_l, bands)
    allowed = np.tril(np.ones((N, N), dtype=bool)) if causal else np.ones((N, N), dtype=bool)

    # RMS(Xbar) over the whole head and over each band (one scalar per head)
    rms_q = {"full": rms(Qb)}
    rms_k = {"full": rms(Kb)}
    for z, idx in dims.items():
        rms_q[z] = rms(Qb[:, :, idx]) if len(idx) else np.zeros(h)
        rms_k[z] = rms(Kb[:, :, idx]) if len(idx) else np.zeros(h_kv)

    tau: Dict[str, np.ndarray] = {}
    scale: Dict[str, np.ndarray] = {}
    logits: Dict[str, np.ndarray] = {}
    probs: Dict[str, np.ndarray] = {}
    band_masks: Dict[str, np.ndarray] = {}
    for z, idx in dims.items():
        d_z = len(idx)
        logits[z] = np.full((h, N, N), -np.inf)
        probs[z] = np.zeros((h, N, N))
        band_masks[z] = np.zeros((h, N, N), dtype=bool)
        if d_z == 0:                               # band switched off
            tau[z] = np.full(h, np.nan)
            scale[z] = np.full(h, np.nan)
            continue
        # S_z = softmax( Qbar_z Kbar_z^T / (sqrt(d_z) tau_z) ), tau_z from the band energies
        tau[z] = (temperature(d_z, d, rms_q[z], rms_q["full"], rms_k[z][kv_of], rms_k["full"][kv_of])
                  if calibrate else np.ones(h))
        scale[z] = np.sqrt(d_z) * tau[z]
        for hq in range(h):
            Qz, Kz = Qb[hq][:, idx], Kb[kv_of[hq]][:, idx]
            usable = np.isfinite(scale[z][hq]) and scale[z][hq] > 0.0
            l = Qz @ Kz.T / scale[z][hq] if usable else np.zeros((N, N))   # no band energy: flat
            logits[z][hq] = np.where(allowed, l, -np.inf)
            probs[z][hq] = softmax_rows(logits[z][hq])
            chosen = np.ones((N, N), dtype=bool) if p >= 1.0 else top_p(probs[z][hq], p)
            band_masks[z][hq] = chosen & allowed

    mask = band_masks["high"] | band_masks["low"]
    forced = np.zeros((h, N, N), dtype=bool)
    if force_diagonal:
        forced[:, np.arange(N), np.arange(N)] = True
    if force_sink:
        forced[:, :, 0] = True
    mask = mask | forced
    return Selection(mask, band_masks, logits, probs, tau, scale, Qb, Kb, rms_q, rms_k,
                     allowed, forced)


def mask_to_csr(mask: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """[h, N, N] bool -> (row_ptr int32 [h*N+1], col_idx int32 [nnz]); one row per
    (head, q-block), columns ascending."""
    h, N, _ = mask.shape
    flat = mask.reshape(h * N, N)
    counts = flat.sum(axis=1)
    row_ptr = np.zeros(h * N + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    col_idx = np.nonzero(flat)[1].astype(np.int32)
    return row_ptr.astype(np.int32), col_idx


@dataclass
class Tolerance:
    """Per-block verdict classes for comparing another implementation's mask."""
    must: np.ndarray        # [h, N, N] bool — has to be selected
    must_not: np.ndarray    # [h, N, N] bool — has to be unselected
    valid: np.ndarray       # [N, N] bool — block pairs open to selection
    # everything else is "don't care"

    @property
    def dont_care_fraction(self) -> float:
        h = self.must.shape[0]
        dc = (~self.must) & (~self.must_not) & self.valid[None]
        return float(dc.sum()) / float(h * self.valid.sum())


def selection_tolerance(sel: Selection, p: float, logit_margin: float = 1e-3,
                        p_margin: float = 2e-5) -> Tolerance:
    """Blocks whose selection may legitimately differ in another implementation.

    Per band and row the selected set is the top-k* blocks by score, the cutoff lying
    between the lowest selected score l_in and the highest unselected score l_out.  A
    block is "don't care" when
      - it is selected and its score is within `logit_margin` of l_out, or it is
        unselected and within `logit_margin` of l_in (a score error of that size could
        swap it across the cutoff; exact ties fall here too), or
      - it enters the set somewhere between p - p_margin and p + p_margin: the taken mass
        at the cutoff is so close to p that fp32 arithmetic decides differently from fp64.
        p_margin is sized for an implementation whose logits are within 2e-5 + 4e-6 |l| of
        these (1.2e-4 at |l| = 25): the mass share A / (A + B) of a top set then moves by at
        most A B / (A + B)^2 * 2 * 1.2e-4 <= 1.2e-5 near p = 0.95, plus about 2e-6 of fp32
        rounding in the exponentials and their sums.
    must = union over bands of (selected minus don't-care); must_not = complement of the
    union over bands of (selected or don't-care)."""
    h, N, _ = sel.mask.shape
    tri = sel.valid[None]
    keep = np.zeros((h, N, N), dtype=bool)       # union_z (M_z \ D_z)
    cover = np.zeros((h, N, N), dtype=bool)      # union_z (M_z | D_z)
    for z in ("high", "low"):
        mz, lz, pz = sel.band_masks[z], sel.logits[z], sel.probs[z]
        if not mz.any():
            continue
        l_in = np.where(mz, lz, np.inf).min(axis=-1, keepdims=True)
        l_out = np.where((~mz) & tri, lz, -np.inf).max(axis=-1, keepdims=True)
        with np.errstate(invalid="ignore"):
            swap_out = mz & ((lz - l_out) <= logit_margin)
            swap_in = (~mz) & tri & ((l_in - lz) <= logit_margin)
        if p >= 1.0:
            shell = np.zeros_like(mz)
        else:
            hi = top_p(pz, p + p_margin) if p + p_margin < 1.0 else np.broadcast_to(tri, mz.shape)
            lo = top_p(pz, max(p - p_margin, 1e-12))
            shell = hi & ~lo
        dz = (swap_out | swap_in | shell) & tri
        keep |= mz & ~dz
        cover |= (mz | dz)
    keep |= sel.forced
    cover |= sel.forced
    return Tolerance(must=keep, must_not=(~cover) | (~tri), valid=sel.valid)


# --------------------------------------------------------------------------- #
# Part 2 — attention by its plain definition
# --------------------------------------------------------------------------- #
def block_sparse_attention_row(Qh: np.ndarray, Kh: np.ndarray, Vh: np.ndarray,
                               u: int, blocks: Sequence[int], B: int, causal: bool = True
                               ) -> Tuple[np.ndarray, np.ndarray]:
    """One q-block of one head.  For token i in block u the visible set is
    J(i) = { j <= i : block(j) in `blocks` } (without `j <= i` when causal is False);
    o_i = sum_J softmax_J(q_i.k_j/sqrt(d)) v_j.
    Qh/Kh/Vh: [L, d] fp64.  Returns (O [rows, d], lse [rows]); a token with an empty
    visible set gets a zero output row and lse = -inf."""
    L, d = Qh.shape
    r0, r1 = u * B, min(L, (u + 1) * B)
    rows = np.arange(r0, r1)
    if len(blocks) == 0:
        return np.zeros((r1 - r0, d)), np.full(r1 - r0, -np.inf)
    cols = np.concatenate([np.arange(v * B, min(L, (v + 1) * B)) for v in blocks])
    s = (Qh[r0:r1] @ Kh[cols].T) / np.sqrt(d)
    if causal:
        s = np.where(cols[None, :] <= rows[:, None], s, -np.inf)
    m = s.max(axis=1, keepdims=True)
    out = np.zeros((r1 - r0, d))
    lse = np.full(r1 - r0, -np.inf)
    ok = np.isfinite(m[:, 0])
    e = np.exp(s[ok] - m[ok])
    den = e.sum(axis=1, keepdims=True)
    out[ok] = (e / den) @ Vh[cols]
    lse[ok] = m[ok, 0] + np.log(den[:, 0])
    return out, lse


def block_sparse_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, mask: np.ndarray,
                           B: int, rows: Optional[Sequence[Tuple[int, int]]] = None,
                           causal: bool = True
                           ) -> Dict[Tuple[int, int], Tuple[np.ndarray, np.ndarray]]:
    """Block-masked attention (causal unless causal=False) for the listed (head, q-block)
    rows (all rows when `rows` is None).  Q: [h, L, d]; K, V: [h_kv, L, d];
    mask: [h, N, N] bool."""
    h, L, d = Q.shape
    g = h // K.shape[0]
    N = mask.shape[1]
    if rows is None:
        rows = [(hq, u) for hq in range(h) for u in range(N)]
    out = {}
    for hq, u in rows:
        blocks = np.nonzero(mask[hq, u, :u + 1] if causal else mask[hq, u])[0]
        out[(hq, u)] = block_sparse_attention_row(Q[hq], K[hq // g], V[hq // g], u, blocks, B,
                                                  causal)
    return out


def dense_causal_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray,
                           q_chunk: int = 1024) -> Tuple[np.ndarray, np.ndarray]:
    """softmax(Q K^T / sqrt(d) + causal) V over whole heads.  Returns
    (O [h, L, d], lse [h, L]).  Query rows are processed in chunks only to bound
    memory; each chunk sees all keys."""
    h, L, d = Q.shape
    g = h // K.shape[0]
    O = np.empty((h, L, d))
    lse = np.empty((h, L))
    j = np.arange(L)
    for hq in range(h):
        Kh, Vh = K[hq // g], V[hq // g]
        for r0 in range(0, L, q_chunk):
            r1 = min(L, r0 + q_chunk)
            s = (Q[hq, r0:r1] @ Kh[:r1].T) / np.sqrt(d)
            s = np.where(j[None, :r1] <= np.arange(r0, r1)[:, None], s, -np.inf)
            m = s.max(axis=1, keepdims=True)
            e = np.exp(s - m)
            den = e.sum(axis=1, keepdims=True)
            O[hq, r0:r1] = (e / den) @ Vh[:r1]
            lse[hq, r0:r1] = m[:, 0] + np.log(den[:, 0])
    return O, lse


def dense_full_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray
                         ) -> Tuple[np.ndarray, np.ndarray]:
    """softmax(Q K^T / sqrt(d)) V with every key visible to every query
    (bidirectional attention).  Returns (O [h, L, d], lse [h, L])."""
    h, L, d = Q.shape
    g = h // K.shape[0]
    O = np.empty((h, L, d))
    lse = np.empty((h, L))
    for hq in range(h):
        s = (Q[hq] @ K[hq // g].T) / np.sqrt(d)
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)
        den = e.sum(axis=1, keepdims=True)
        O[hq] = (e / den) @ V[hq // g]
        lse[hq] = m[:, 0] + np.log(den[:, 0])
    return O, lse
