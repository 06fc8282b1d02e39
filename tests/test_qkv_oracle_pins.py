"""Pins of the QKV-projection + rotary-embedding oracle against facts it does not compute itself:
a hand-worked 2-dimensional rotation, exact integer products, the identity weight, norm
preservation, and the relative-position property of the rotary embedding."""
import math

import numpy as np

from oracle.qkv_oracle import qkv_rope, rope_tables


def test_two_dimensional_head_is_a_plane_rotation():
    # d = 2: one pair; angle(p, 0) = p.  y = (3, 4) rotated by 90 degrees is (-4, 3).
    x = np.array([[1.0]])
    w = np.array([[3.0], [4.0], [5.0], [6.0], [7.0], [8.0]])      # one Q, one K, one V head of width 2
    cos_t = np.array([[1.0], [math.cos(math.pi / 2)]])
    sin_t = np.array([[0.0], [math.sin(math.pi / 2)]])
    q, k, v = qkv_rope(x, w, cos_t, sin_t, [1], 1, 1, 2)
    np.testing.assert_allclose(q[0, 0], [-4.0, 3.0], atol=1e-15)
    np.testing.assert_allclose(k[0, 0], [-6.0, 5.0], atol=1e-15)
    np.testing.assert_allclose(v[0, 0], [7.0, 8.0], atol=0)        # V is not rotated


def test_position_zero_is_the_plain_projection_exact_in_integers():
    rng = np.random.default_rng(5)
    T, Hin, hq, hkv, d = 5, 7, 3, 2, 4
    x = rng.integers(-4, 5, (T, Hin))
    w = rng.integers(-4, 5, ((hq + 2 * hkv) * d, Hin))
    cos_t, sin_t = rope_tables(3, d)
    q, k, v = qkv_rope(x, w, cos_t, sin_t, np.zeros(T, dtype=int), hq, hkv, d)
    want = np.zeros((T, (hq + 2 * hkv) * d), dtype=np.int64)
    for t in range(T):                       # brute force, integer arithmetic
        for f in range(want.shape[1]):
            want[t, f] = sum(int(x[t, c]) * int(w[f, c]) for c in range(Hin))
    got = np.concatenate([q.reshape(T, -1), k.reshape(T, -1), v.reshape(T, -1)], axis=1)
    assert np.array_equal(got, want.astype(np.float64))


def test_identity_weight_hands_the_input_through_in_head_order():
    hq, hkv, d = 2, 1, 4
    n = (hq + 2 * hkv) * d
    x = np.arange(3 * n, dtype=np.float64).reshape(3, n)
    cos_t, sin_t = rope_tables(2, d)
    q, k, v = qkv_rope(x, np.eye(n), cos_t, sin_t, [0, 0, 0], hq, hkv, d)
    assert np.array_equal(q.reshape(3, -1), x[:, :hq * d])
    assert np.array_equal(k.reshape(3, -1), x[:, hq * d:(hq + hkv) * d])
    assert np.array_equal(v.reshape(3, -1), x[:, (hq + hkv) * d:])
    # a transposed weight or a K/V swap would permute these columns


def test_rotation_keeps_norms_and_pairs_i_with_i_plus_half():
    rng = np.random.default_rng(6)
    T, Hin, hq, hkv, d = 6, 9, 2, 2, 8
    x = rng.standard_normal((T, Hin))
    w = rng.standard_normal(((hq + 2 * hkv) * d, Hin))
    cos_t, sin_t = rope_tables(50, d)
    pos = np.array([0, 3, 7, 11, 30, 49])
    q, k, v = qkv_rope(x, w, cos_t, sin_t, pos, hq, hkv, d)
    q0, k0, v0 = qkv_rope(x, w, cos_t, sin_t, np.zeros(T, dtype=int), hq, hkv, d)
    np.testing.assert_allclose(np.linalg.norm(q, axis=-1), np.linalg.norm(q0, axis=-1), rtol=1e-13)
    np.testing.assert_allclose(np.linalg.norm(k, axis=-1), np.linalg.norm(k0, axis=-1), rtol=1e-13)
    assert np.array_equal(v, v0)
    # each (i, i + d/2) pair keeps its own norm: the rotation does not mix pairs
    h = d // 2
    np.testing.assert_allclose(q[..., :h] ** 2 + q[..., h:] ** 2, q0[..., :h] ** 2 + q0[..., h:] ** 2, rtol=1e-12)
    # and pair i turns by angle pos * base**(-2i/d): check pair 1 of token 2 by hand
    ang = 7 * 10000.0 ** (-2.0 / d)
    a, b = q0[2, 0, 1], q0[2, 0, 1 + h]
    np.testing.assert_allclose([q[2, 0, 1], q[2, 0, 1 + h]],
                               [a * math.cos(ang) - b * math.sin(ang), b * math.cos(ang) + a * math.sin(ang)], rtol=1e-13)


def test_scores_depend_on_the_position_difference_only():
    rng = np.random.default_rng(7)
    Hin, d = 5, 16
    x = rng.standard_normal((2, Hin))
    w = rng.standard_normal((3 * d, Hin))
    cos_t, sin_t = rope_tables(200, d)

    def score(pq, pk):
        q, k, _ = qkv_rope(x, w, cos_t, sin_t, [pq, pk], 1, 1, d)
        return float(q[0, 0] @ k[1, 0])

    np.testing.assert_allclose(score(17, 5), score(112, 100), rtol=1e-12)
    np.testing.assert_allclose(score(3, 3), score(150, 150), rtol=1e-12)
    assert abs(score(17, 5) - score(17, 6)) > 1e-6   # and it does depend on that difference


def test_output_projection_is_the_plain_product_exact_in_integers():
    from oracle.qkv_oracle import o_proj
    rng = np.random.default_rng(8)
    T, hq, d, nout = 4, 2, 3, 5
    o = rng.integers(-5, 6, (T, hq, d))
    w = rng.integers(-5, 6, (nout, hq * d))
    want = np.zeros((T, nout), dtype=np.int64)
    for t in range(T):
        for f in range(nout):
            want[t, f] = sum(int(o[t, h, i]) * int(w[f, h * d + i]) for h in range(hq) for i in range(d))
    assert np.array_equal(o_proj(o, w), want.astype(np.float64))
    # heads are concatenated in order: a weight that picks element (h, i) returns it
    pick = np.zeros((1, hq * d)); pick[0, 1 * d + 2] = 1.0
    assert np.array_equal(o_proj(o, pick)[:, 0], o[:, 1, 2].astype(np.float64))
