"""Oracle of the producer in front of the training-time-test attention: the draft layer's query /
key / value projection followed by the rotary position embedding, written in the layout the
attention kernels read (Sec. 4.2.1 takes Q_j, K_j, V_j of every TTT step as given; this is the op
that makes them).  TEST INFRASTRUCTURE: plain numpy in fp64, the definition written out; only
tests, the smoke check and the benchmarks' cpu_baseline legs may use it.

    y[t, f]   = sum_c x[t, c] * w[f, c]                    f over (hq + 2 hkv) heads of width d
    Q, K heads: for i < d/2, with c = cos_tab[pos[t], i], s = sin_tab[pos[t], i]
                out[i]       = y[i] * c - y[i + d/2] * s
                out[i + d/2] = y[i + d/2] * c + y[i] * s
    V heads:    out = y

Readings (the paper does not spell this op out; they follow the model families it trains drafts
for): no bias; the weight is stored [out_features, in_features] with the Q heads first, then the K
heads, then the V heads; the rotation pairs element i with element i + d/2 of a head ("rotate
half"); the angle table is an input, indexed by a per-token position id, so the choice of base
frequency and of the position ids of a TTT step stays with the caller.
"""
import numpy as np


def rope_tables(n_pos, d, base=10000.0):
    """cos, sin of shape [n_pos, d/2] in fp64: angle(p, i) = p * base**(-2 i / d)."""
    inv = base ** (-np.arange(0, d, 2, dtype=np.float64) / d)
    ang = np.arange(n_pos, dtype=np.float64)[:, None] * inv[None, :]
    return np.cos(ang), np.sin(ang)


def qkv_rope(x, w, cos_tab, sin_tab, pos, hq, hkv, d):
    """x [T, Hin], w [(hq + 2 hkv) d, Hin], cos_tab / sin_tab [n_pos, d/2], pos [T] ->
    q [T, hq, d], k [T, hkv, d], v [T, hkv, d], all fp64."""
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    T = x.shape[0]
    assert w.shape == ((hq + 2 * hkv) * d, x.shape[1]) and d % 2 == 0
    y = (x @ w.T).reshape(T, hq + 2 * hkv, d)
    c = np.asarray(cos_tab, dtype=np.float64)[np.asarray(pos)][:, None, :]   # [T, 1, d/2]
    s = np.asarray(sin_tab, dtype=np.float64)[np.asarray(pos)][:, None, :]
    h = d // 2

    def rot(u):
        lo, hi = u[..., :h], u[..., h:]
        return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)

    return rot(y[:, :hq]), rot(y[:, hq:hq + hkv]), y[:, hq + hkv:].copy()


def o_proj(o, w):
    """The consumer on the other side of the attention: out[t, f] = sum_c o[t, c] * w[f, c], with o the
    attention output [T, hq, d] (or already [T, hq * d]) and w [out_features, hq * d]; fp64."""
    o = np.asarray(o, dtype=np.float64)
    o = o.reshape(o.shape[0], -1)
    w = np.asarray(w, dtype=np.float64)
    assert w.shape[1] == o.shape[1]
    return o @ w.T
