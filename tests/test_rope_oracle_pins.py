"""Pins of the rotary-embedding reference (oracle/rope_oracle.py) against what the mathematics
fixes: identity at position 0, a hand-worked rotation, norm preservation, the relative-position
property that is the point of the embedding (RoFormer Eq. 16: the score of a rotated query and key
depends on the distance only), composition of rotations, inverse = transpose, the complex-number
form of the same rotation, and packed = unpacked (the position reset)."""
import numpy as np

from oracle import rope_oracle as ro


def rnd(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_hand_worked_rotation():
    # d = 4, base 100: inverse frequencies 1 and 0.1; the row at local position 2 turns by 2 and 0.2 rad
    x = np.zeros((3, 1, 4)); x[2, 0] = [1.0, 2.0, 3.0, 4.0]
    y = ro.rope_packed(x, [0, 3], base=100.0)
    want = [1 * np.cos(2) - 3 * np.sin(2), 2 * np.cos(0.2) - 4 * np.sin(0.2),
            3 * np.cos(2) + 1 * np.sin(2), 4 * np.cos(0.2) + 2 * np.sin(0.2)]
    assert np.allclose(y[2, 0], want, atol=1e-15)
    assert np.allclose(y[2, 0], [-3.1440390, 1.1654559, -0.3391431, 4.3176045], atol=1e-6)   # by calculator


def test_position_zero_is_identity_and_every_sequence_starts_there():
    x = rnd((10, 2, 8), 1)
    cu = [0, 4, 4, 9, 10]
    y = ro.rope_packed(x, cu)
    for start in (0, 4, 9):
        assert np.array_equal(y[start], x[start])
    assert not np.allclose(y[5], x[5])


def test_norms_are_preserved_pairwise():
    x = rnd((50, 3, 16), 2)
    y = ro.rope_packed(x, [0, 50])
    assert np.allclose(x[..., :8] ** 2 + x[..., 8:] ** 2, y[..., :8] ** 2 + y[..., 8:] ** 2, atol=1e-12)


def test_scores_depend_on_distance_only():
    d = 16
    q, k = rnd((1, 1, d), 3), rnd((1, 1, d), 4)
    def score(m, n):
        L = max(m, n) + 1
        Q = np.zeros((L, 1, d)); K = np.zeros((L, 1, d)); Q[m] = q[0]; K[n] = k[0]
        return float(ro.rope_packed(Q, [0, L])[m, 0] @ ro.rope_packed(K, [0, L])[n, 0])
    assert abs(score(7, 3) - score(104, 100)) < 1e-11
    assert abs(score(5, 5) - float(q[0, 0] @ k[0, 0])) < 1e-12
    assert abs(score(7, 3) - score(3, 7)) > 1e-3                       # the sign of the distance matters


def test_inverse_is_the_transpose_and_undoes_the_rotation():
    x, g = rnd((30, 2, 8), 5), rnd((30, 2, 8), 6)
    cu = [0, 11, 30]
    y = ro.rope_packed(x, cu)
    assert np.allclose(ro.rope_packed(y, cu, inverse=True), x, atol=1e-12)
    # <R x, g> = <x, R^T g>: the inverse carries gradients
    assert abs(float((y * g).sum()) - float((x * ro.rope_packed(g, cu, inverse=True)).sum())) < 1e-10


def test_complex_form():
    # the same rotation written as multiplication of x[i] + j x[i + d/2] by exp(j m theta_i)
    x = rnd((20, 1, 8), 7)
    y = ro.rope_packed(x, [0, 20], base=500.0)
    z = x[:, 0, :4] + 1j * x[:, 0, 4:]
    theta = 500.0 ** (-2.0 * np.arange(4) / 8)
    w = z * np.exp(1j * np.arange(20)[:, None] * theta[None, :])
    assert np.allclose(y[:, 0, :4], w.real, atol=1e-12) and np.allclose(y[:, 0, 4:], w.imag, atol=1e-12)


def test_packed_equals_unpacked():
    lengths = [5, 1, 0, 9]
    cu = np.concatenate([[0], np.cumsum(lengths)])
    x = rnd((int(cu[-1]), 2, 8), 8)
    y = ro.rope_packed(x, cu)
    for s, L in enumerate(lengths):
        a = int(cu[s])
        assert np.array_equal(y[a:a + L], ro.rope_packed(x[a:a + L], [0, L]))
