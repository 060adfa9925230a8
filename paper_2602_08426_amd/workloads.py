"""Seeded synthetic Q/K/V workloads for the Prism hot path.

This module only *makes inputs*: post-RoPE bf16 query/key/value tensors with the
head geometry, RoPE bases and qualitative attention structure (sink, local
window, slash lines, vertical stripes, heavy-tailed key norms) of long-context
LLM prefill, which is the setting of the paper's efficiency experiment
(Sec. 4.3 "Efficiency Results", Fig. "Efficiency comparison").  It holds none of
the method's arithmetic (no pooling, scoring, selection or attention): both the
CPU oracle's tests and the GPU binding's tests/bench consume the bits produced
here, and neither the oracle nor the HIP path imports the other.

RoPE follows the paper's Sec. 3.1 "Spectral Structure of RoPE": feature pair j
is the adjacent dims (2j, 2j+1), rotated by angle n * theta_j at position n with
theta_j = base ** (-2j/d).

All tensors are returned as numpy uint16 arrays holding bf16 bit patterns
(round-to-nearest-even applied exactly once), layout [heads, seq_len, head_dim].
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np


# --------------------------------------------------------------------------- #
# bf16 bit helpers (input packing only)
# --------------------------------------------------------------------------- #
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 -> bf16 (nearest even), return the 16-bit patterns as uint16."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- #
# RoPE (input generator side)
# --------------------------------------------------------------------------- #
def rope_frequencies(head_dim: int, base: float, yarn=None) -> np.ndarray:
    """theta_j = base^(-2j/d), j = 0 .. d/2-1 (fp64).  yarn = (native_len, scale, alpha, beta)
    stretches the low frequencies the way a YaRN-extended checkpoint does (NTK-by-parts: pairs that
    turn fewer than alpha times over native_len are slowed by `scale`, pairs that turn more than
    beta times are kept, linear blend between)."""
    j = np.arange(head_dim // 2, dtype=np.float64)
    theta = np.power(float(base), -2.0 * j / head_dim)
    if yarn is not None:
        native_len, scale, alpha, beta = yarn
        turns = native_len * theta / (2.0 * np.pi)
        keep = np.clip((turns - alpha) / (beta - alpha), 0.0, 1.0)
        theta = (1.0 - keep) * theta / scale + keep * theta
    return theta


def rope_tables(positions: np.ndarray, head_dim: int, base: float, yarn=None) -> Tuple[np.ndarray, np.ndarray]:
    """cos/sin of n*theta_j as fp32 [len(positions), d/2]; angles formed in fp64."""
    ang = positions.astype(np.float64)[:, None] * rope_frequencies(head_dim, base, yarn)[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def apply_rope(x: np.ndarray, cos: np.ndarray, sin: np.ndarray) -> np.ndarray:
    """Rotate adjacent pairs (2j, 2j+1) of x [L, d] by the tabulated angles."""
    out = np.empty_like(x)
    xe, xo = x[:, 0::2], x[:, 1::2]
    out[:, 0::2] = xe * cos - xo * sin
    out[:, 1::2] = xe * sin + xo * cos
    return out


def rotate_vector(g: np.ndarray, shift: float, head_dim: int, base: float, yarn=None) -> np.ndarray:
    """R_shift g: rotate a single content vector by `shift` positions (fp64)."""
    th = rope_frequencies(head_dim, base, yarn) * float(shift)
    c, s = np.cos(th), np.sin(th)
    out = np.empty(head_dim, dtype=np.float64)
    out[0::2] = g[0::2] * c - g[1::2] * s
    out[1::2] = g[0::2] * s + g[1::2] * c
    return out


# --------------------------------------------------------------------------- #
# Workload descriptions
# --------------------------------------------------------------------------- #
@dataclass(frozen=True)
class Workload:
    name: str
    n_q_heads: int
    n_kv_heads: int
    seq_len: int
    block: int
    rope_base: float
    top_p: float
    seed: int
    recipe: str                      # which per-head role mix to plant
    head_dim: int = 128
    d_high: int = 64
    d_low: int = 96
    k_lognormal_sigma: float = 0.0   # heavy-tailed per-token key scales (0 = off)
    amp_scale: float = 1.0           # multiplies the planted q-side amplitudes (density knob)
    yarn: Optional[Tuple[int, float, float, float]] = None   # (native_len, scale, alpha, beta): YaRN-style frequencies
    noise_topic_amp: float = 0.3     # topic amplitude of the near-noise heads (their density knob)

    @property
    def n_blocks(self) -> int:
        return -(-self.seq_len // self.block)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


WORKLOADS: Dict[str, Workload] = {
    # 1 head, 2K tokens, block 64, slash at offset 16 + sink at token 0.
    "c1_2k_slash": Workload("c1_2k_slash", 1, 1, 2048, 64, 1.0e4, 0.95, 1000, "slash16"),
    # Llama-3-8B-shaped layer (32 q / 8 kv heads, base 5e5), 8K tokens.
    "c2_llama_8k": Workload("c2_llama_8k", 32, 8, 8192, 128, 5.0e5, 0.95, 1001, "mixed",
                            amp_scale=0.8),
    # Same layer at 32K.
    "c3_llama_32k": Workload("c3_llama_32k", 32, 8, 32768, 128, 5.0e5, 0.95, 1002, "mixed",
                             amp_scale=0.7),
    # Same layer at 128K: the configuration the headline metric is quoted on.
    "c4_llama_128k": Workload("c4_llama_128k", 32, 8, 131072, 128, 5.0e5, 0.95, 1003, "mixed",
                              amp_scale=0.6),
    # Qwen2.5-7B-shaped layer (28 q / 4 kv heads, base 1e6), 64K, heavy-tailed K norms.
    "c5_qwen_64k": Workload("c5_qwen_64k", 28, 4, 65536, 128, 1.0e6, 0.93, 1004, "mixed",
                            k_lognormal_sigma=0.75, amp_scale=0.55),
    # The 128K layer at block 64 (N = 2048, the largest block count the library takes): the
    # block-size study of the paper's appendix; same tokens as c4, not a headline configuration.
    "c4_llama_128k_b64": Workload("c4_llama_128k_b64", 32, 8, 131072, 64, 5.0e5, 0.95, 1003, "mixed",
                                  amp_scale=0.6),
}


def small_variant(w: Workload, seq_len: int, n_q_heads: int | None = None,
                  n_kv_heads: int | None = None, block: int | None = None) -> Workload:
    """Same recipe and geometry family at a reduced size (parity-test cases)."""
    return Workload(
        name=f"{w.name}@{seq_len}", n_q_heads=n_q_heads or w.n_q_heads,
        n_kv_heads=n_kv_heads or w.n_kv_heads, seq_len=seq_len, block=block or w.block,
        rope_base=w.rope_base, top_p=w.top_p, seed=w.seed, recipe=w.recipe,
        head_dim=w.head_dim, d_high=w.d_high, d_low=w.d_low,
        k_lognormal_sigma=w.k_lognormal_sigma, amp_scale=w.amp_scale,
        noise_topic_amp=w.noise_topic_amp)


@dataclass
class HeadPlan:
    """What is planted in one q-head (q side) — for reporting only."""
    role: str
    slash_offsets: List[int] = field(default_factory=list)
    slash_amp: float = 0.0
    vert_amp: float = 0.0
    topic_amp: float = 1.0        # amplitude of the q side's block-level topic vectors


@dataclass
class KVPlan:
    """What is planted in one kv-head (k side)."""
    g_amp: float
    stripe_blocks: np.ndarray
    stripe_amp: float
    sink_amp: float
    topic_amp: float


# Amplitudes (and each workload's amp_scale) were tuned once against the CPU oracle so
# that top-p selection at the workload's p keeps roughly 5-15% of the causal block
# pairs at 32K-128K; they are frozen here together with the seeds.
# Role of q-head i in the "mixed" recipe: local / slash / vertical / mixed in turn, and every
# sixteenth head (i % 16 == 15) a near-noise head whose weak structure leaves the block-level
# distribution flat, so that top-p keeps almost every causal block (measured 0.92 - 0.97 of them).
# A full quarter of such heads would put the layer's density at 0.3, outside the 0.05 - 0.15 the
# benchmark configurations ask for; one in sixteen keeps the layer inside it and still exercises
# the long, high-entropy rows.
_ROLE_TABLE = ("local", "slash", "vertical", "mixed")
_NOISE_EVERY = 16
_SLASH_CHOICES = (16, 100, 1000, 5000)


def _plan(w: Workload) -> Tuple[List[HeadPlan], List[KVPlan], np.ndarray, np.ndarray]:
    """Draw the per-head planted structure from the workload seed."""
    rng = np.random.default_rng(np.random.SeedSequence([w.seed, 0xA11CE]))
    d, nb = w.head_dim, w.n_blocks
    g_vecs = rng.standard_normal((w.n_kv_heads, d))          # stationary content per kv head
    # semantic direction lives in the slowest-rotating dims (last 16)
    m_vecs = np.zeros((w.n_kv_heads, d))
    m_vecs[:, d - 16:] = rng.standard_normal((w.n_kv_heads, 16))
    m_vecs /= np.linalg.norm(m_vecs, axis=1, keepdims=True) / 4.0   # |m| = 4

    kv_plans: List[KVPlan] = []
    for _ in range(w.n_kv_heads):
        n_stripes = max(1, int(round(0.01 * nb)))
        stripes = np.sort(rng.choice(np.arange(nb), size=min(nb, n_stripes), replace=False))
        kv_plans.append(KVPlan(g_amp=1.0, stripe_blocks=stripes,
                               stripe_amp=float(rng.uniform(2.5, 3.5)),
                               sink_amp=float(rng.uniform(5.0, 7.0)),
                               topic_amp=float(rng.uniform(1.0, 2.0))))

    head_plans: List[HeadPlan] = []
    if w.recipe == "slash16":
        head_plans = [HeadPlan("slash", [16], 3.0, 1.0) for _ in range(w.n_q_heads)]
    elif w.recipe == "mixed":
        for hq in range(w.n_q_heads):
            role = "noise" if hq % _NOISE_EVERY == _NOISE_EVERY - 1 else _ROLE_TABLE[hq % 4]
            if role == "local":
                hp = HeadPlan(role, [0, w.block // 2, w.block], float(rng.uniform(2.0, 3.0)),
                              float(rng.uniform(0.5, 1.0)))
            elif role == "slash":
                offs = [o for o in _SLASH_CHOICES if o < w.seq_len // 2]
                o = int(rng.choice(offs))
                hp = HeadPlan(role, [0, o], float(rng.uniform(2.0, 3.0)),
                              float(rng.uniform(0.5, 1.0)))
            elif role == "vertical":
                hp = HeadPlan(role, [0], float(rng.uniform(1.0, 1.5)),
                              float(rng.uniform(2.0, 3.0)))
            elif role == "mixed":
                offs = [o for o in _SLASH_CHOICES if o < w.seq_len // 2]
                o = int(rng.choice(offs))
                hp = HeadPlan(role, [0, o], float(rng.uniform(1.5, 2.5)),
                              float(rng.uniform(1.5, 2.5)))
            else:
                offs = [o for o in _SLASH_CHOICES if o < w.seq_len // 2]
                rng.choice(offs)                       # same number of draws as the role it replaces
                hp = HeadPlan(role, [0], float(rng.uniform(0.2, 0.5)), float(rng.uniform(0.1, 0.3)),
                              topic_amp=w.noise_topic_amp)
            head_plans.append(hp)
    else:
        raise ValueError(f"unknown recipe {w.recipe!r}")
    for hp in head_plans:
        hp.slash_amp *= w.amp_scale
        hp.vert_amp *= w.amp_scale
    return head_plans, kv_plans, g_vecs, m_vecs


_Q_TOPIC_AMP = 1.0
_TOPIC_DIMS = 32


def _add_block_topics(x: np.ndarray, rng: np.random.Generator, B: int, d: int, amp: float) -> None:
    """Block-level semantic content: every token of a block shares one random vector in
    the slowest-rotating dims, so that block-level scores vary from block to block (the
    'block-sparse pattern' of semantic heads) instead of being flat."""
    L = x.shape[0]
    nb = -(-L // B)
    t = rng.standard_normal((nb, _TOPIC_DIMS), dtype=np.float32) * np.float32(amp)
    x[:, d - _TOPIC_DIMS:] += np.repeat(t, B, axis=0)[:L]


def describe(w: Workload) -> List[dict]:
    """Per-q-head planted roles (for reports)."""
    hp, _, _, _ = _plan(w)
    return [dict(head=i, role=p.role, slash_offsets=p.slash_offsets,
                 slash_amp=round(p.slash_amp, 3), vert_amp=round(p.vert_amp, 3))
            for i, p in enumerate(hp)]


def generate(w: Workload, n_threads: int = 8, rotate: bool = True) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Return (Q, K, V) as bf16 bit patterns (uint16), shapes
    [n_q_heads, L, d], [n_kv_heads, L, d], [n_kv_heads, L, d].  rotate=False returns Q and K as
    they are BEFORE the rotary embedding (rounded to bf16), for callers that apply it themselves."""
    L, d, B = w.seq_len, w.head_dim, w.block
    head_plans, kv_plans, g_vecs, m_vecs = _plan(w)
    cos, sin = rope_tables(np.arange(L), d, w.rope_base, w.yarn)
    if not rotate:
        cos, sin = np.ones_like(cos), np.zeros_like(sin)
    root = np.random.SeedSequence([w.seed, 0xDA7A])
    seeds = root.spawn(w.n_q_heads + 2 * w.n_kv_heads)

    Q = np.empty((w.n_q_heads, L, d), dtype=np.uint16)
    K = np.empty((w.n_kv_heads, L, d), dtype=np.uint16)
    V = np.empty((w.n_kv_heads, L, d), dtype=np.uint16)

    def make_q(hq: int) -> None:
        rng = np.random.default_rng(seeds[hq])
        kvh = hq // w.group
        hp = head_plans[hq]
        x = rng.standard_normal((L, d), dtype=np.float32)
        const = hp.vert_amp * m_vecs[kvh]
        for o in hp.slash_offsets:
            const = const + (hp.slash_amp / np.sqrt(len(hp.slash_offsets))) * \
                rotate_vector(g_vecs[kvh], -o, d, w.rope_base, w.yarn)
        x += const.astype(np.float32)[None, :]
        _add_block_topics(x, rng, B, d, _Q_TOPIC_AMP * hp.topic_amp)
        Q[hq] = f32_to_bf16_bits(apply_rope(x, cos, sin))

    def make_k(kvh: int) -> None:
        rng = np.random.default_rng(seeds[w.n_q_heads + kvh])
        kp = kv_plans[kvh]
        x = rng.standard_normal((L, d), dtype=np.float32)
        x += (kp.g_amp * g_vecs[kvh]).astype(np.float32)[None, :]
        mv = m_vecs[kvh].astype(np.float32)
        for b in kp.stripe_blocks:
            x[b * B:(b + 1) * B] += kp.stripe_amp * mv[None, :]
        x[0] += kp.sink_amp * mv
        _add_block_topics(x, rng, B, d, kp.topic_amp)
        if w.k_lognormal_sigma > 0.0:
            z = rng.standard_normal(L, dtype=np.float32)
            x *= np.exp(np.float32(w.k_lognormal_sigma) * z)[:, None]
        K[kvh] = f32_to_bf16_bits(apply_rope(x, cos, sin))

    def make_v(kvh: int) -> None:
        rng = np.random.default_rng(seeds[w.n_q_heads + w.n_kv_heads + kvh])
        V[kvh] = f32_to_bf16_bits(rng.standard_normal((L, d), dtype=np.float32))

    jobs = [(make_q, i) for i in range(w.n_q_heads)] + \
           [(make_k, i) for i in range(w.n_kv_heads)] + \
           [(make_v, i) for i in range(w.n_kv_heads)]
    if n_threads <= 1:
        for fn, i in jobs:
            fn(i)
    else:
        with ThreadPoolExecutor(max_workers=n_threads) as ex:
            list(ex.map(lambda fi: fi[0](fi[1]), jobs))
    return Q, K, V


def constant_content_rope(content: np.ndarray, positions: np.ndarray, base: float) -> np.ndarray:
    """fp64 [len(positions), d]: the same content vector placed at each position and
    rotated by RoPE — the stationary-content case of the paper's Sec. 3.2."""
    d = content.shape[0]
    ang = positions.astype(np.float64)[:, None] * rope_frequencies(d, base)[None, :]
    c, s = np.cos(ang), np.sin(ang)
    out = np.empty((len(positions), d), dtype=np.float64)
    out[:, 0::2] = content[0::2][None, :] * c - content[1::2][None, :] * s
    out[:, 1::2] = content[0::2][None, :] * s + content[1::2][None, :] * c
    return out
