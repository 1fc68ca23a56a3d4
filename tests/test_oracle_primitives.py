"""Pins of the oracle's building blocks against library routines and closed forms."""
import numpy as np
import scipy.special
import torch

from oracle import goose_oracle as orc

RNG = np.random.default_rng(1234)


def test_rmsnorm_matches_library():
    x = RNG.standard_normal((5, 48)) * 3.0
    g = 1.0 + 0.3 * RNG.standard_normal(48)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), 1e-5).numpy()
    np.testing.assert_allclose(orc.rmsnorm(x, g, 1e-5), ref, rtol=1e-12, atol=1e-12)


def test_rmsnorm_unit_rms_and_eps():
    x = RNG.standard_normal((3, 64))
    y = orc.rmsnorm(x, np.ones(64), 0.0)
    np.testing.assert_allclose(np.sqrt((y * y).mean(-1)), 1.0, rtol=1e-12)
    # eps matters for a tiny row: x*rsqrt(x^2+eps) with one element
    y = orc.rmsnorm(np.array([[1e-3]]), np.ones(1), 1e-5)
    np.testing.assert_allclose(y, [[1e-3 / np.sqrt(1e-6 + 1e-5)]], rtol=1e-12)


def test_silu_and_softmax_match_library():
    x = RNG.standard_normal(100) * 4
    np.testing.assert_allclose(orc.silu(x), torch.nn.functional.silu(torch.from_numpy(x)).numpy(), rtol=1e-12)
    s = RNG.standard_normal((4, 9)) * 5
    np.testing.assert_allclose(orc.softmax_rows(s), scipy.special.softmax(s, axis=-1), rtol=1e-12)


def test_attention_matches_library_with_mask():
    T, S, n_h, d = 6, 11, 3, 16
    q = RNG.standard_normal((T, n_h, d))
    K = RNG.standard_normal((n_h, S, d))
    V = RNG.standard_normal((n_h, S, d))
    allow = RNG.random((T, S)) < 0.6
    allow[:, 0] = True
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).permute(1, 0, 2)[None], torch.from_numpy(K)[None], torch.from_numpy(V)[None],
        attn_mask=torch.from_numpy(allow)[None, None])[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(orc.attention(q, K, V, allow), ref, rtol=1e-10, atol=1e-12)


def test_rope_closed_form_complex_rotation():
    T, n_h, d, base = 7, 2, 8, 10000.0
    x = RNG.standard_normal((T, n_h, d))
    pos = np.array([0, 1, 2, 5, 17, 100, 1023])
    y = orc.rope(x, pos, base)
    half = d // 2
    for j in range(half):
        z = (x[..., j] + 1j * x[..., j + half]) * np.exp(1j * pos[:, None] * base ** (-2.0 * j / d))
        np.testing.assert_allclose(y[..., j], z.real, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(y[..., j + half], z.imag, rtol=1e-12, atol=1e-12)
    # position 0 is the identity, norms are preserved
    np.testing.assert_allclose(y[0], x[0])
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-12)


def test_rope_scores_depend_on_relative_position_only():
    d, base = 16, 10000.0
    q = RNG.standard_normal((1, 1, d))
    k = RNG.standard_normal((1, 1, d))
    def score(m, n):
        return float(orc.rope(q, [m], base)[0, 0] @ orc.rope(k, [n], base)[0, 0])
    np.testing.assert_allclose(score(9, 4), score(105, 100), rtol=1e-10)
    np.testing.assert_allclose(score(9, 4), score(5, 0), rtol=1e-10)
    assert abs(score(9, 4) - score(4, 9)) > 1e-6  # the sign of the offset matters


def test_argmax_lowest_index_on_ties_and_margin():
    l = np.array([[1.0, 3.0, 3.0, 2.0], [5.0, 5.0, 5.0, 5.0], [0.0, -1.0, 7.0, 6.5]])
    assert orc.argmax_lowest(l).tolist() == [1, 0, 2]
    np.testing.assert_allclose(orc.top2_margin(l), [0.0, 0.0, 0.5])
