"""Pins for the oracle's elementary operations against closed forms and torch CPU library routines."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import dflash_oracle as O


def test_round_bf16_matches_torch_cast():
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(4096) * 10.0 ** rng.integers(-6, 6, 4096),
                        # exact halfway cases between neighbouring bf16 values (ties-to-even)
                        np.array([1.00390625, 1.01171875, -3.0078125, 0.0, 2.0 ** -20])])
    got = O.round_bf16(x)
    ref = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(got, ref)
    assert O.round_bf16(np.array([1.00390625]))[0] == 1.0          # tie -> even (down)
    assert O.round_bf16(np.array([1.01171875]))[0] == 1.015625     # tie -> even (up)


def test_round_bf16_pair_is_two_bf16_numbers_with_sixteen_bits():
    """hi + lo storage of a GEMM input: hi and lo are each representable in bf16 (checked against torch's cast, not
    against the oracle's own rounding), hi is the nearest bf16 to x, lo the nearest bf16 to the fp32 remainder, and the
    pair is within 2^-16 |x| of x (two 8-bit significands less the overlap); a value with at most 16 significant bits
    that are split evenly is reproduced exactly."""
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.integers(-6, 6, 4000), [0.0, 1.0, -1.0, 3.0e-5, 65280.0]])
    x = x.astype(np.float32).astype(np.float64)
    r = O.round_bf16_pair(x)
    xt = torch.from_numpy(x.astype(np.float32))
    hi = xt.to(torch.bfloat16).to(torch.float32)
    lo = (xt - hi).to(torch.bfloat16).to(torch.float32)
    assert np.array_equal(r, hi.double().numpy() + lo.double().numpy())
    lo_o = torch.from_numpy((r - hi.double().numpy()).astype(np.float32))
    assert torch.equal(lo_o.to(torch.bfloat16).to(torch.float32), lo_o)          # what is left beside hi is one bf16 number
    assert (np.abs(x - r) <= 2.0 ** -16 * np.abs(x)).all()
    assert np.abs(x - r).max() > 0                                               # and it is a rounding, not the identity
    exact = np.array([1.0 + 2.0 ** -7 + 2.0 ** -14, 3.0 - 2.0 ** -13, -(2.0 ** 20 + 2.0 ** 6)])
    assert np.array_equal(O.round_bf16_pair(exact), exact)
    single = O.round_bf16(x)
    assert np.abs(x - single).max() / np.abs(x - r).max() > 50                   # the pair is far finer than one bf16 number


def test_rmsnorm_library_and_scale_invariance():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((5, 96))
    g = rng.uniform(0.5, 1.5, 96)
    got = O.rmsnorm(x, g, 1e-6)
    ref = F.rms_norm(torch.from_numpy(x), (96,), torch.from_numpy(g), 1e-6).numpy()
    assert np.allclose(got, ref, rtol=1e-12, atol=1e-12)
    # RMSNorm(alpha x) == RMSNorm(x) when eps is negligible
    assert np.allclose(O.rmsnorm(7.5 * x, g, 0.0), O.rmsnorm(x, g, 0.0), rtol=1e-12)
    # unit gain, eps 0 -> rows have unit mean square
    assert np.allclose(np.mean(O.rmsnorm(x, np.ones(96), 0.0) ** 2, -1), 1.0)


def test_rope_equals_complex_rotation():
    rng = np.random.default_rng(3)
    T, H, hd, theta = 7, 3, 64, 1e4
    x = rng.standard_normal((T, H, hd))
    pos = np.array([0, 1, 2, 17, 300, 4095, 16383])
    got = O.rope(x, pos, theta)
    z = x[..., : hd // 2] + 1j * x[..., hd // 2:]
    freq = np.array([theta ** (-(2 * i) / hd) for i in range(hd // 2)])
    zr = z * np.exp(1j * pos[:, None, None] * freq[None, None, :])
    assert np.allclose(got[..., : hd // 2], zr.real, atol=1e-9)
    assert np.allclose(got[..., hd // 2:], zr.imag, atol=1e-9)
    assert np.array_equal(got[0], x[0])                                 # position 0 is identity
    assert np.allclose(np.linalg.norm(got, axis=-1), np.linalg.norm(x, axis=-1))


def test_rope_scores_depend_on_position_difference_only():
    rng = np.random.default_rng(4)
    q = rng.standard_normal((1, 1, 128))
    k = rng.standard_normal((1, 1, 128))
    for theta in (1e4, 1e6):
        s0 = (O.rope(q, np.array([40]), theta) * O.rope(k, np.array([33]), theta)).sum()
        s1 = (O.rope(q, np.array([1040]), theta) * O.rope(k, np.array([1033]), theta)).sum()
        s2 = (O.rope(q, np.array([41]), theta) * O.rope(k, np.array([33]), theta)).sum()
        assert abs(s0 - s1) < 1e-9
        assert abs(s0 - s2) > 1e-3


def test_softmax_and_silu_library():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((4, 33)) * 5
    assert np.allclose(O.softmax(x), torch.softmax(torch.from_numpy(x), -1).numpy(), atol=1e-15)
    assert np.allclose(O.silu(x), F.silu(torch.from_numpy(x)).numpy(), atol=1e-14)
    # no overflow for large scores
    assert np.isfinite(O.softmax(np.array([[1e4, 0.0, -1e4]]))).all()


class _M:
    n_q_heads, n_kv_heads, head_dim = 8, 2, 16


def test_attend_matches_sdpa_with_gqa():
    rng = np.random.default_rng(6)
    n = 37
    q = rng.standard_normal((_M.n_q_heads, _M.head_dim))
    K = rng.standard_normal((n, _M.n_kv_heads, _M.head_dim))
    V = rng.standard_normal((n, _M.n_kv_heads, _M.head_dim))
    got = O._attend(_M, q, K, V)
    tq = torch.from_numpy(q)[None, :, None, :]                           # [1, Hq, 1, hd]
    tk = torch.from_numpy(K).permute(1, 0, 2)[None].repeat_interleave(4, dim=1)
    tv = torch.from_numpy(V).permute(1, 0, 2)[None].repeat_interleave(4, dim=1)
    ref = F.scaled_dot_product_attention(tq, tk, tv)[0, :, 0, :].numpy()
    assert np.allclose(got, ref, atol=1e-12)


def test_counter_uniform_is_uniform_and_keyed():
    from scipy import stats
    idx = np.arange(200000)
    u = O.counter_uniform(12345, 3, 5, 0, idx)
    assert u.min() > 0.0 and u.max() < 1.0
    counts = np.histogram(u, bins=64, range=(0, 1))[0]
    assert stats.chisquare(counts).pvalue > 1e-4
    # lag-1 correlation and stream separation
    assert abs(np.corrcoef(u[:-1], u[1:])[0, 1]) < 0.01
    for other in (O.counter_uniform(12346, 3, 5, 0, idx), O.counter_uniform(12345, 4, 5, 0, idx),
                  O.counter_uniform(12345, 3, 6, 0, idx), O.counter_uniform(12345, 3, 5, 1, idx)):
        assert abs(np.corrcoef(u, other)[0, 1]) < 0.01
    # worked value of the stated recipe, computed with Python integers
    key, seq, slot, purpose, i = 99, 2, 7, 1, 1234
    M = (1 << 64) - 1
    c = ((((seq * 64 + slot) * 4 + purpose) << 32) | i)
    z = (key + 0x9E3779B97F4A7C15 * (c + 1)) & M
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M
    z = z ^ (z >> 31)
    assert O.counter_uniform(key, seq, slot, purpose, np.array([i]))[0] == ((z >> 41) + 0.5) / 2 ** 23


def test_gumbel_argmax_samples_the_softmax():
    from scipy import stats
    logw = np.log(np.array([0.5, 0.25, 0.125, 0.0625, 0.0625]))
    counts = np.zeros(5)
    n = 20000
    for k in range(n):
        counts[int(np.argmax(O.gumbel_scores(logw, 1000 + k, 0, 1, 0)))] += 1
    assert stats.chisquare(counts, n * np.exp(logw)).pvalue > 1e-4


def test_appendix_a3_memory_figures():
    """Sizes printed in Appendix A.3 (KV injection: memory overhead), from tests/golden."""
    import os
    vals = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "appendix_a3_memory.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split("=")
                vals[k.strip()] = float(v)
    m = O.fusion_memory_bytes(d_model=2048, n_taps=5, seq_len=2048, block_size=16)
    assert m["w_c"] == 5 * 2048 * 2048 * 2
    assert abs(m["w_c"] / 1e6 - vals["w_c_MB"]) < 0.5
    assert abs(m["proj_in"] / 1e6 - vals["proj_in_MB"]) < 2.5       # "about 40 MB"
    assert abs(m["proj_out"] / 1e6 - vals["proj_out_MB"]) < 0.5     # "8 MB"
    assert m["decode_tmp"] < vals["decode_tmp_max_KB"] * 1000
