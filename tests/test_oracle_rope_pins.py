"""Pins of the rotary-embedding oracle (positions re-used across contexts, Section 1 of arXiv
2502.05431; the rotation itself is the published rotary position embedding, half-split pairing)."""
import math

import numpy as np
import pytest
import torch

from oracle import ape_oracle


def _x(n, heads, d, seed=0):
    return np.random.default_rng(seed).standard_normal((n, heads, d)).astype(np.float32)


def test_against_complex_multiplication():
    """The rotation of the plane (x_c, x_{c+d/2}) by the angle pos * base^(-2c/d) IS the complex
    product (x_c + i x_{c+d/2}) * exp(i angle): numpy's complex arithmetic computes it with no
    rotation formula written out here (and nothing of the product package is involved)."""
    lens, off, base = [5, 9, 1, 12], 8, 500000.0
    d = 64
    x = _x(sum(lens), 3, d, 1)
    pos = np.concatenate([off + np.arange(l) for l in lens]).astype(np.float64)
    freq = np.float64(base) ** (-np.arange(d // 2, dtype=np.float64) * 2.0 / d)
    z = (x[..., :d // 2].astype(np.float64) + 1j * x[..., d // 2:].astype(np.float64)) * np.exp(1j * pos[:, None, None] * freq[None, None, :])
    ref = np.concatenate([z.real, z.imag], axis=-1)
    got = ape_oracle.rope(x, lens, off, base)
    np.testing.assert_allclose(got, ref, atol=1e-13)
    assert torch.tensor(got).shape == (sum(lens), 3, d)


def test_position_zero_is_identity_and_planes_keep_their_norm():
    x = _x(7, 2, 32, 2)
    y = ape_oracle.rope(x, [1] * 7, 0, 10000.0)            # seven one-token segments, all at position 0
    np.testing.assert_array_equal(y, x.astype(np.float64))
    y = ape_oracle.rope(x, [7], 3, 10000.0)
    n_in = x[..., :16].astype(np.float64) ** 2 + x[..., 16:].astype(np.float64) ** 2
    n_out = y[..., :16] ** 2 + y[..., 16:] ** 2
    np.testing.assert_allclose(n_out, n_in, rtol=1e-13)


def test_base_one_turns_every_plane_by_the_position_in_radians():
    """base = 1: all planes turn by `pos` radians; checked against math.cos/sin directly."""
    x = _x(4, 1, 8, 3)
    y = ape_oracle.rope(x, [4], 2, 1.0)
    for j in range(4):
        c, s = math.cos(2 + j), math.sin(2 + j)
        for k in range(4):
            x1, x2 = float(x[j, 0, k]), float(x[j, 0, k + 4])
            assert y[j, 0, k] == pytest.approx(x1 * c - x2 * s, abs=1e-15)
            assert y[j, 0, k + 4] == pytest.approx(x2 * c + x1 * s, abs=1e-15)


def test_scores_depend_on_the_position_difference_only():
    """The defining property of the rotary embedding: <R_m q, R_n k> = <R_(m-n) q, k>."""
    d, base = 64, 500000.0
    q, k = _x(1, 1, d, 4), _x(1, 1, d, 5)
    for m, n in ((17, 5), (1000, 993), (40, 40)):
        qm = ape_oracle.rope(q, [1], m, base)[0, 0]
        kn = ape_oracle.rope(k, [1], n, base)[0, 0]
        qd = ape_oracle.rope(q, [1], m - n, base)[0, 0]
        assert qm @ kn == pytest.approx(qd @ k[0, 0].astype(np.float64), abs=1e-10)


def test_frequencies_per_plane():
    """Plane c turns by pos * base^(-2c/d): a unit vector in plane c comes back as (cos, sin)."""
    d, base, pos = 16, 10000.0, 11
    x = np.zeros((1, 1, d), np.float32)
    x[0, 0, :8] = 1.0
    y = ape_oracle.rope(x, [1], pos, base)[0, 0]
    for c in range(8):
        a = pos * base ** (-2.0 * c / d)
        assert y[c] == pytest.approx(math.cos(a), abs=1e-14)
        assert y[c + 8] == pytest.approx(math.sin(a), abs=1e-14)


def test_positions_restart_in_every_context():
    lens, off = [6, 3, 6], 32
    x = _x(15, 2, 32, 6)
    x[6:9] = x[0:3]
    x[9:15] = x[0:6]
    y = ape_oracle.rope(x, lens, off, 500000.0)
    np.testing.assert_array_equal(y[6:9], y[0:3])
    np.testing.assert_array_equal(y[9:15], y[0:6])
    # ... and differ from one long sequence
    z = ape_oracle.rope(x, [15], off, 500000.0)
    assert np.abs(z[9:15] - y[9:15]).max() > 1e-2


def test_bad_arguments():
    with pytest.raises(ValueError):
        ape_oracle.rope(_x(2, 1, 7), [2], 0, 10000.0)      # odd head_dim
    with pytest.raises(ValueError):
        ape_oracle.rope(_x(2, 1, 8), [2], 0, 0.0)
