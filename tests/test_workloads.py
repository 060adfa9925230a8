"""Host-side checks of the synthetic input generator (no GPU)."""
import numpy as np
import torch

from paper_2602_08426_amd import workloads as wl


def test_bf16_rounding_matches_torch_rne():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(100000).astype(np.float32) * 37.0,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38], np.float32)])
    got = wl.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(got, ref)
    np.testing.assert_array_equal(wl.bf16_bits_to_f32(got),
                                  torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_rope_preserves_norm_and_relative_position():
    d, base = 128, 5.0e5
    rng = np.random.default_rng(1)
    a, b = rng.standard_normal(d), rng.standard_normal(d)
    pos = np.array([5, 105, 1005, 1105])
    A = wl.constant_content_rope(a, pos, base)
    Bm = wl.constant_content_rope(b, pos, base)
    np.testing.assert_allclose(np.linalg.norm(A, axis=1), np.linalg.norm(a), rtol=1e-12)
    # <R_m a, R_n b> depends on m - n only
    assert abs(A[1] @ Bm[0] - A[3] @ Bm[2]) < 1e-9
    # fp32 table path agrees with the fp64 path
    cos, sin = wl.rope_tables(pos, d, base)
    x = np.repeat(a[None].astype(np.float32), len(pos), 0)
    np.testing.assert_allclose(wl.apply_rope(x, cos, sin), A, atol=2e-6)


def test_generate_is_deterministic_and_shaped():
    w = wl.small_variant(wl.WORKLOADS["c5_qwen_64k"], 1024, 7, 1)
    q1, k1, v1 = wl.generate(w, n_threads=1)
    q2, k2, v2 = wl.generate(w, n_threads=4)
    assert q1.shape == (7, 1024, 128) and k1.shape == (1, 1024, 128) and v1.shape == (1, 1024, 128)
    assert q1.dtype == np.uint16
    np.testing.assert_array_equal(q1, q2)
    np.testing.assert_array_equal(k1, k2)
    np.testing.assert_array_equal(v1, v2)
    assert np.isfinite(wl.bf16_bits_to_f32(k1)).all()


def test_all_baseline_configs_present():
    names = ["c1_2k_slash", "c2_llama_8k", "c3_llama_32k", "c4_llama_128k", "c5_qwen_64k"]
    assert list(wl.WORKLOADS)[:5] == names
    b64 = wl.WORKLOADS["c4_llama_128k_b64"]                # the 128K layer at block 64 (N = 2048)
    assert (b64.seq_len, b64.block, b64.n_blocks, b64.seed) == (131072, 64, 2048, 1003)
    c4 = wl.WORKLOADS["c4_llama_128k"]
    assert (c4.n_q_heads, c4.n_kv_heads, c4.seq_len, c4.block, c4.n_blocks) == (32, 8, 131072, 128, 1024)
    c5 = wl.WORKLOADS["c5_qwen_64k"]
    assert (c5.n_q_heads, c5.n_kv_heads, c5.top_p, c5.rope_base) == (28, 4, 0.93, 1.0e6)


def test_generator_and_oracle_agree_on_the_rope_convention():
    """Two independent implementations (the generator's tables, the oracle's complex rotation) of the
    same convention: pairs (2j, 2j+1), angle n * theta_j, plain and YaRN-scaled frequencies."""
    import dataclasses

    from oracle import prism_oracle as orc
    yarn = (32768, 4.0, 1.0, 32.0)
    np.testing.assert_allclose(wl.rope_frequencies(128, 1.0e6, yarn), orc.rope_frequencies(128, 1.0e6, yarn=yarn),
                               rtol=1e-14)
    for y in (None, yarn):
        w = dataclasses.replace(wl.small_variant(wl.WORKLOADS["c5_qwen_64k"], 512, 2, 1), yarn=y)
        q_pre, k_pre, v0 = wl.generate(w, n_threads=1, rotate=False)
        q_rot, k_rot, v1 = wl.generate(w, n_threads=1)
        np.testing.assert_array_equal(v0, v1)
        theta = orc.rope_frequencies(w.head_dim, w.rope_base, yarn=y)
        for pre, rot in ((q_pre, q_rot), (k_pre, k_rot)):
            # the generator rotates its fp32 content before rounding; rotating the rounded pre-RoPE
            # tensor instead differs by the rounding of the content (2^-9 relative per element)
            ref = orc.apply_rope(orc.bf16_to_f64(pre), theta)
            got = orc.bf16_to_f64(rot)
            scale = np.abs(orc.bf16_to_f64(pre)).max()
            assert np.abs(got - ref).max() < 2.0 ** -6 * scale
