"""Pins for the oracle's building blocks: closed forms, special cases, library routines."""
import math

import numpy as np
import pytest
import torch

from .helpers import dp, f32, fp


def test_bf16_round_matches_library_conversion(orc):
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * s for s in (1e-3, 1.0, 300.0)])
    got = np.array([orc.orc_bf16_round(float(v)) for v in x], np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).float().numpy()
    assert np.array_equal(got, want)


def test_bf16_round_ties_to_even(orc):
    # 1 + 2^-8 is exactly half way between bf16 neighbours 1 and 1 + 2^-7: even mantissa wins
    assert orc.orc_bf16_round(1.0 + 2.0 ** -8) == 1.0
    assert orc.orc_bf16_round(1.0 + 2.0 ** -7 + 2.0 ** -8) == 1.0 + 2.0 ** -6
    assert orc.orc_bf16_round(1.0 + 2.0 ** -8 + 2.0 ** -20) == 1.0 + 2.0 ** -7
    assert orc.orc_bf16_round(-0.0) == 0.0


@pytest.mark.parametrize("y,k", [(-3.2, 0), (0.49, 0), (0.5, 0), (0.51, 1), (1.5, 2), (2.5, 2), (3.5, 4),
                                 (7.6, 8), (8.4, 8), (99.0, 8), (-0.5, 0), (float("nan"), 0)])
def test_round_clamp_table(orc, y, k):
    # Eq. 3: round (half to even), then min(k_max, max(0, .))
    assert orc.orc_round_clamp(y, 8) == k


def test_round_clamp_other_kmax(orc):
    assert orc.orc_round_clamp(9.7, 10) == 10
    assert orc.orc_round_clamp(9.4, 10) == 9
    assert orc.orc_round_clamp(5.0, 0) == 0


def test_argmax_lowest_index_wins(orc):
    x = f32([0.0, 3.0, -1.0, 3.0, 2.0])
    assert orc.orc_argmax(fp(x), 5) == 1
    x = f32([-5.0])
    assert orc.orc_argmax(fp(x), 1) == 0


def test_rmsnorm_constant_vector(orc):
    d, c, eps = 64, -3.0, 1e-6
    g = f32(np.linspace(0.5, 2.0, d))
    out = np.zeros(d, np.float32)
    orc.orc_rmsnorm(fp(f32(np.full(d, c))), fp(g), d, eps, fp(out))
    np.testing.assert_allclose(out, g * c / math.sqrt(c * c + eps), rtol=1e-6)


def test_rmsnorm_unit_rms_and_scale_invariance(orc):
    rng = np.random.default_rng(1)
    d = 256
    x = f32(rng.standard_normal(d) * 7)
    g = f32(np.ones(d))
    a, b = np.zeros(d, np.float32), np.zeros(d, np.float32)
    orc.orc_rmsnorm(fp(x), fp(g), d, 0.0, fp(a))
    orc.orc_rmsnorm(fp(f32(x * 4)), fp(g), d, 0.0, fp(b))
    assert abs(np.sqrt(np.mean(a.astype(np.float64) ** 2)) - 1.0) < 1e-6
    np.testing.assert_allclose(a, b, rtol=1e-6)


def test_rope_position_zero_is_identity(orc):
    rng = np.random.default_rng(2)
    x = f32(rng.standard_normal(4 * 64))
    y = x.copy()
    orc.orc_rope(fp(y), 4, 64, 0, 10000.0)
    assert np.array_equal(x, y)


def test_rope_head_dim_two_is_a_plane_rotation(orc):
    # with head_dim 2 the single frequency is base^0 = 1: rotation by `pos` radians
    for pos in (1, 2, 7):
        y = f32([1.0, 0.0, 0.0, 1.0])  # two heads
        orc.orc_rope(fp(y), 2, 2, pos, 10000.0)
        np.testing.assert_allclose(y, [math.cos(pos), math.sin(pos), -math.sin(pos), math.cos(pos)], atol=1e-6)


def test_rope_frequencies_and_pairing(orc):
    # one-hot at index i (first half) lands on (i, i+half) with angle pos * base^(-2i/hd)
    hd, half, base, pos = 8, 4, 100.0, 3
    for i in range(half):
        x = np.zeros(hd, np.float32)
        x[i] = 1.0
        orc.orc_rope(fp(x), 1, hd, pos, base)
        ang = pos * base ** (-2.0 * i / hd)
        want = np.zeros(hd)
        want[i], want[i + half] = math.cos(ang), math.sin(ang)
        np.testing.assert_allclose(x, want, atol=1e-6)


def test_rope_relative_position_property(orc):
    rng = np.random.default_rng(3)
    hd = 64
    q, k = f32(rng.standard_normal(hd)), f32(rng.standard_normal(hd))

    def dot(m, n):
        a, b = q.copy(), k.copy()
        orc.orc_rope(fp(a), 1, hd, m, 10000.0)
        orc.orc_rope(fp(b), 1, hd, n, 10000.0)
        assert abs(np.linalg.norm(a) - np.linalg.norm(q)) < 1e-4
        return float(a.astype(np.float64) @ b.astype(np.float64))
    assert abs(dot(5, 2) - dot(13, 10)) < 1e-4
    assert abs(dot(40, 40) - float(q.astype(np.float64) @ k.astype(np.float64))) < 1e-4
    assert abs(dot(5, 2) - dot(2, 5)) > 1e-3  # not symmetric: sign of the angle matters


def _attn(orc, q, k, v, H, Hk, hd):
    out = np.zeros(H * hd, np.float32)
    orc.orc_attention_row(fp(q), fp(k), fp(v), k.shape[0], H, Hk, hd, Hk * hd, fp(out))
    return out


def test_attention_single_key_returns_value(orc):
    rng = np.random.default_rng(4)
    H, hd = 3, 16
    q, k, v = (f32(rng.standard_normal((1, H * hd))) for _ in range(3))
    np.testing.assert_allclose(_attn(orc, q[0], k, v, H, H, hd), v[0], rtol=1e-6)


def test_attention_equal_scores_gives_mean(orc):
    rng = np.random.default_rng(5)
    H, hd, n = 2, 8, 11
    q = f32(rng.standard_normal(H * hd))
    k = f32(np.tile(rng.standard_normal((1, H * hd)), (n, 1)))
    v = f32(rng.standard_normal((n, H * hd)))
    np.testing.assert_allclose(_attn(orc, q, k, v, H, H, hd), v.mean(0), rtol=1e-5, atol=1e-6)


@pytest.mark.parametrize("H,Hk", [(4, 4), (8, 2), (4, 1)])
def test_attention_matches_library_sdpa_float64(orc, H, Hk):
    rng = np.random.default_rng(6)
    hd, n = 32, 37
    q = f32(rng.standard_normal(H * hd))
    k = f32(rng.standard_normal((n, Hk * hd)))
    v = f32(rng.standard_normal((n, Hk * hd)))
    got = _attn(orc, q, k, v, H, Hk, hd)
    tq = torch.from_numpy(q).double().view(H, 1, hd)
    g = H // Hk
    tk = torch.from_numpy(k).double().view(n, Hk, hd).permute(1, 0, 2).repeat_interleave(g, 0)
    tv = torch.from_numpy(v).double().view(n, Hk, hd).permute(1, 0, 2).repeat_interleave(g, 0)
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).reshape(-1).numpy()
    np.testing.assert_allclose(got, want, rtol=2e-5, atol=2e-6)


def test_attention_gqa_head_mapping(orc):
    # one key; V differs per KV head, so the output tells which KV head each query head read
    H, Hk, hd = 8, 2, 4
    q = f32(np.ones(H * hd))
    k = f32(np.ones((1, Hk * hd)))
    v = f32(np.concatenate([np.full(hd, 10.0), np.full(hd, 20.0)])[None])
    out = _attn(orc, q, k, v, H, Hk, hd).reshape(H, hd)
    assert np.all(out[:4] == 10.0) and np.all(out[4:] == 20.0)


def test_attention_scale_is_inverse_sqrt_head_dim(orc):
    # two keys with scores +-s: weights are softmax([s, -s] / sqrt(hd))
    hd = 16
    q = f32(np.ones(hd))
    k = f32(np.stack([np.ones(hd) * 0.5, -np.ones(hd) * 0.5]))
    v = f32(np.stack([np.ones(hd), np.zeros(hd)]))
    out = _attn(orc, q, k, v, 1, 1, hd)
    s = 0.5 * hd / math.sqrt(hd)
    np.testing.assert_allclose(out, 1.0 / (1.0 + math.exp(-2 * s)), rtol=1e-6)


def test_inverse_cdf_table(orc):
    q = np.array([0.0, 0.2, 0.0, 0.5, 0.3], np.float64)
    for u, want in [(0.0, 1), (0.19, 1), (0.2, 3), (0.69, 3), (0.7, 4), (0.999999, 4)]:
        assert orc.orc_sample_inverse_cdf(dp(q), 5, u) == want
    q2 = q * 7.5  # unnormalised input gives the same answer
    assert orc.orc_sample_inverse_cdf(dp(q2), 5, 0.69) == 3
    # u so close to 1 that u * total rounds to the total: the draw must still carry mass
    q3 = np.array([0.25, 0.75, 0.0, 0.0], np.float64)
    for u in (1.0, float(np.nextafter(1.0, 0.0))):
        assert orc.orc_sample_inverse_cdf(dp(q3), 4, u) == 1
