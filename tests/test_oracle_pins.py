"""Pins of the fp64 oracle against things other than itself (CPU only).

What the paper and the mathematics fix: Alg. 2's printed predicate, a library attention routine
(torch SDPA, fp64) for the special cases that reduce to it, finite differences, closed forms,
invariants, and a brute-force evaluation on tiny inputs.
"""
import itertools
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import ttt_dense

RNG = np.random.default_rng(20260318)


def rand_inputs(k, T, hq, hkv, d, dtype=np.float64, with_do=True):
    Q = RNG.standard_normal((k, T, hq, d)).astype(dtype)
    K = RNG.standard_normal((k, T, hkv, d)).astype(dtype)
    V = RNG.standard_normal((k, T, hkv, d)).astype(dtype)
    dO = RNG.standard_normal((k, T, hq, d)).astype(dtype) if with_do else None
    return Q, K, V, dO


# ---------------------------------------------------------------- mask (Alg. 2)
def alg2_flat(q_i, kv_i, q_len, seq_len):
    """Alg. 2 exactly as printed, on flat indices of one padded sequence."""
    m_causal = q_i >= kv_i
    m_pad = kv_i < seq_len
    M_causal = m_causal and m_pad
    m_suffix = kv_i >= q_len
    m_pad = (kv_i % q_len) < seq_len
    m_diag = ((kv_i - q_i) % q_len) == 0
    M_suffix = m_suffix and m_pad and m_diag
    return M_causal or M_suffix


@pytest.mark.parametrize("q_len,seq_len,k", [(1, 1, 3), (4, 4, 1), (5, 3, 4), (7, 7, 4), (6, 5, 2)])
def test_alg2_predicate_equals_step_position_predicate(oracle, q_len, seq_len, k):
    """Brute force: for real (unpadded) query rows i < T, Alg. 2 on flat indices, restricted to the
    j+1 blocks in the cache at step j, equals the oracle's (block, token) predicate on a document
    of length T."""
    M = oracle.oracle_mask(k, [0, seq_len])                 # [k*T, k*T] from the C predicate
    for j, i in itertools.product(range(k), range(seq_len)):
        for l, m_pos in itertools.product(range(k), range(q_len)):
            kv_i = l * q_len + m_pos
            in_cache = l <= j
            want = in_cache and alg2_flat(i, kv_i, q_len, seq_len)
            if m_pos >= seq_len:
                assert not want                                  # pad keys are never visible
                continue
            assert bool(M[j * seq_len + i, l * seq_len + m_pos]) == want, (j, i, l, m_pos)


@pytest.mark.parametrize("k,cu", [(3, [0, 5, 6, 13]), (2, [0, 0, 4, 4, 9]), (4, [0, 1, 2, 3])])
def test_packed_mask_matches_dense_alg2(oracle, k, cu):
    assert np.array_equal(oracle.oracle_mask(k, cu), ttt_dense.packed_mask(k, cu))
    M = oracle.oracle_mask(k, cu)
    T = cu[-1]
    starts = np.repeat(np.array(cu[:-1]), np.diff(cu))
    # visible-key count per row: (i - start + 1) + j
    for j in range(k):
        for i in range(T):
            assert M[j * T + i].sum() == (i - starts[i] + 1) + j


# ---------------------------------------------------------------- library routine pins
def sdpa_concat(Q, K, V, M, scale, dO=None):
    """torch fp64 SDPA on the concatenated k*T sequence with an explicit boolean mask."""
    k, T, hq, d = Q.shape
    hkv = K.shape[2]
    G = hq // hkv
    q = torch.tensor(Q.reshape(k * T, hq, d)).permute(1, 0, 2)[None].clone().requires_grad_(True)
    kk = torch.tensor(K.reshape(k * T, hkv, d)).permute(1, 0, 2)[None].clone().requires_grad_(True)
    vv = torch.tensor(V.reshape(k * T, hkv, d)).permute(1, 0, 2)[None].clone().requires_grad_(True)
    kr = kk.repeat_interleave(G, dim=1)
    vr = vv.repeat_interleave(G, dim=1)
    o = F.scaled_dot_product_attention(q, kr, vr, attn_mask=torch.tensor(M)[None, None], scale=scale)
    out = {"O": o[0].permute(1, 0, 2).reshape(k, T, hq, d).detach().numpy()}
    if dO is not None:
        go = torch.tensor(dO.reshape(k * T, hq, d)).permute(1, 0, 2)[None]
        o.backward(go)
        out["dQ"] = q.grad[0].permute(1, 0, 2).reshape(k, T, hq, d).numpy()
        out["dK"] = kk.grad[0].permute(1, 0, 2).reshape(k, T, hkv, d).numpy()
        out["dV"] = vv.grad[0].permute(1, 0, 2).reshape(k, T, hkv, d).numpy()
    return out


def test_k1_is_ordinary_causal_attention(oracle):
    """k = 1: the TTT mask is the causal mask; compare with torch SDPA is_causal per document."""
    cu = [0, 9, 10, 23]
    hq, hkv, d = 4, 2, 8
    Q, K, V, dO = rand_inputs(1, cu[-1], hq, hkv, d)
    scale = 1 / math.sqrt(d)
    O, LSE, dQ, dK, dV = oracle.oracle_full(Q, K, V, cu, scale, dO)
    for a, b in zip(cu[:-1], cu[1:]):
        q = torch.tensor(Q[0, a:b]).permute(1, 0, 2)[None].clone().requires_grad_(True)
        kk = torch.tensor(K[0, a:b]).permute(1, 0, 2)[None].clone().requires_grad_(True)
        vv = torch.tensor(V[0, a:b]).permute(1, 0, 2)[None].clone().requires_grad_(True)
        o = F.scaled_dot_product_attention(q, kk.repeat_interleave(2, 1), vv.repeat_interleave(2, 1),
                                           is_causal=True, scale=scale)
        o.backward(torch.tensor(dO[0, a:b]).permute(1, 0, 2)[None])
        np.testing.assert_allclose(O[0, a:b], o[0].permute(1, 0, 2).detach().numpy(), rtol=0, atol=1e-13)
        np.testing.assert_allclose(dQ[0, a:b], q.grad[0].permute(1, 0, 2).numpy(), rtol=0, atol=1e-13)
        np.testing.assert_allclose(dK[0, a:b], kk.grad[0].permute(1, 0, 2).numpy(), rtol=0, atol=1e-13)
        np.testing.assert_allclose(dV[0, a:b], vv.grad[0].permute(1, 0, 2).numpy(), rtol=0, atol=1e-13)


@pytest.mark.parametrize("k,cu,hq,hkv,d", [(3, [0, 5, 6, 13], 4, 2, 8), (4, [0, 11], 2, 1, 4), (2, [0, 3, 3, 8], 3, 3, 5)])
def test_k_steps_equal_concatenated_sequence_under_block_mask(oracle, k, cu, hq, hkv, d):
    """k steps == one sequence of k*T slots under the explicit mask built from Alg. 2's modular
    predicate; library SDPA fp64 with that boolean mask, and autograd for the backward."""
    Q, K, V, dO = rand_inputs(k, cu[-1], hq, hkv, d)
    scale = 1 / math.sqrt(d)
    M = ttt_dense.packed_mask(k, cu)
    ref = sdpa_concat(Q, K, V, M, scale, dO)
    O, LSE, dQ, dK, dV = oracle.oracle_full(Q, K, V, cu, scale, dO)
    np.testing.assert_allclose(O, ref["O"], rtol=0, atol=1e-13)
    np.testing.assert_allclose(dQ, ref["dQ"], rtol=0, atol=1e-13)
    np.testing.assert_allclose(dK, ref["dK"], rtol=0, atol=1e-13)
    np.testing.assert_allclose(dV, ref["dV"], rtol=0, atol=1e-13)
    # the numpy dense-concatenated form agrees too (and pins LSE)
    Od, LSEd, dQd, dKd, dVd = ttt_dense.dense_forward_backward(Q, K, V, cu, scale, dO)
    np.testing.assert_allclose(O, Od, rtol=0, atol=1e-13)
    np.testing.assert_allclose(LSE, LSEd, rtol=0, atol=1e-13)
    np.testing.assert_allclose(dQ, dQd, rtol=0, atol=1e-13)
    np.testing.assert_allclose(dK, dKd, rtol=0, atol=1e-13)
    np.testing.assert_allclose(dV, dVd, rtol=0, atol=1e-13)


# ---------------------------------------------------------------- brute force on tiny inputs
def brute_force_row(Q, K, V, cu, scale, j, i, h):
    """Pure-Python evaluation of one output row from the (step, position) statement of the mask."""
    hq, hkv = Q.shape[2], K.shape[2]
    g = h // (hq // hkv)
    start = None
    for a, b in zip(cu[:-1], cu[1:]):
        if a <= i < b:
            start = a
    keys = [(0, m) for m in range(start, i + 1)] + [(l, i) for l in range(1, j + 1)]
    s = [scale * float(np.dot(Q[j, i, h], K[l, m, g])) for (l, m) in keys]
    mx = max(s)
    e = [math.exp(x - mx) for x in s]
    z = sum(e)
    o = sum((e_ / z) * V[l, m, g] for e_, (l, m) in zip(e, keys))
    return o, mx + math.log(z), [e_ / z for e_ in e]


def test_brute_force_rows_and_row_sums(oracle):
    k, cu, hq, hkv, d = 3, [0, 4, 5, 9], 4, 2, 3
    Q, K, V, _ = rand_inputs(k, cu[-1], hq, hkv, d, with_do=False)
    scale = 0.7
    O, LSE, *_ = oracle.oracle_full(Q, K, V, cu, scale)
    for j, i, h in itertools.product(range(k), range(cu[-1]), range(hq)):
        o, lse, p = brute_force_row(Q, K, V, cu, scale, j, i, h)
        assert abs(sum(p) - 1.0) < 1e-14
        np.testing.assert_allclose(O[j, i, h], o, rtol=0, atol=1e-14)
        assert abs(LSE[j, h, i] - lse) < 1e-14


def test_rows_of_p_sum_to_one_via_unit_values(oracle):
    """V == 1 everywhere => O == 1 exactly iff every row of P sums to 1."""
    k, cu = 4, [0, 17, 30]
    Q, K, V, _ = rand_inputs(k, cu[-1], 4, 2, 6, with_do=False)
    V[:] = 1.0
    O, *_ = oracle.oracle_full(Q, K, V, cu, 0.5)
    np.testing.assert_allclose(O, 1.0, rtol=0, atol=1e-14)


# ---------------------------------------------------------------- finite differences
def test_backward_matches_central_finite_differences(oracle):
    k, cu, hq, hkv, d = 3, [0, 4, 6], 2, 1, 4
    Q, K, V, dO = rand_inputs(k, cu[-1], hq, hkv, d)
    scale = 1 / math.sqrt(d)
    _, _, dQ, dK, dV = oracle.oracle_full(Q, K, V, cu, scale, dO)

    def loss(Q_, K_, V_):
        O, *_ = oracle.oracle_full(Q_, K_, V_, cu, scale)
        return float((O * dO).sum())

    eps = 1e-5
    for name, X, G in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        num = np.zeros_like(X)
        it = np.nditer(X, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = X[idx]
            X[idx] = old + eps; lp = loss(Q, K, V)
            X[idx] = old - eps; lm = loss(Q, K, V)
            X[idx] = old
            num[idx] = (lp - lm) / (2 * eps)
        err = np.abs(num - G).max() / max(np.abs(G).max(), 1e-30)
        assert err < 1e-7, (name, err)


# ---------------------------------------------------------------- closed forms
def test_closed_form_zero_keys_gives_prefix_means(oracle):
    """K == 0: uniform softmax over (i-start+1)+j keys; pins the key count, the document boundary
    and the query-head -> kv-head map."""
    k, cu, hq, hkv, d = 4, [0, 6, 7, 15], 4, 2, 3
    Q, K, V, _ = rand_inputs(k, cu[-1], hq, hkv, d, with_do=False)
    K[:] = 0.0
    O, LSE, *_ = oracle.oracle_full(Q, K, V, cu, 0.3)
    G = hq // hkv
    for a, b in zip(cu[:-1], cu[1:]):
        for i in range(a, b):
            for j in range(k):
                n = (i - a + 1) + j
                for h in range(hq):
                    g = h // G
                    want = (V[0, a:i + 1, g].sum(axis=0) + V[1:j + 1, i, g].sum(axis=0)) / n
                    np.testing.assert_allclose(O[j, i, h], want, rtol=0, atol=1e-14)
                    assert abs(LSE[j, h, i] - math.log(n)) < 1e-14


def test_closed_form_constant_values(oracle):
    """V_l[m,g,:] == c_g: O == c_{h/G} exactly; dQ == dK == 0."""
    k, cu, hq, hkv, d = 3, [0, 8, 12], 4, 2, 5
    Q, K, V, dO = rand_inputs(k, cu[-1], hq, hkv, d)
    c = RNG.standard_normal((hkv, d))
    V[:] = c[None, None]
    O, _, dQ, dK, dV = oracle.oracle_full(Q, K, V, cu, 0.4, dO)
    for h in range(hq):
        np.testing.assert_allclose(O[:, :, h], np.broadcast_to(c[h // 2], O[:, :, h].shape), rtol=0, atol=1e-14)
    assert np.abs(dQ).max() < 1e-13 and np.abs(dK).max() < 1e-13


def test_closed_form_length_one_documents(oracle):
    """Every document has length 1: row (j,i) is a softmax over exactly K_0[i..],...,K_j[i]."""
    k, T, hq, hkv, d = 4, 5, 2, 1, 3
    cu = list(range(T + 1))
    Q, K, V, _ = rand_inputs(k, T, hq, hkv, d, with_do=False)
    scale = 0.9
    O, LSE, *_ = oracle.oracle_full(Q, K, V, cu, scale)
    for j, i, h in itertools.product(range(k), range(T), range(hq)):
        s = scale * (K[:j + 1, i, 0] @ Q[j, i, h])
        p = np.exp(s - s.max()); p /= p.sum()
        np.testing.assert_allclose(O[j, i, h], p @ V[:j + 1, i, 0], rtol=0, atol=1e-14)


# ---------------------------------------------------------------- invariants of the gradients
def test_gradient_invariants_shift_scale_mass(oracle):
    k, cu, hq, hkv, d = 3, [0, 7, 19], 4, 2, 6
    Q, K, V, dO = rand_inputs(k, cu[-1], hq, hkv, d)
    _, _, dQ, dK, dV = oracle.oracle_full(Q, K, V, cu, 0.35, dO)
    G = hq // hkv
    for a, b in zip(cu[:-1], cu[1:]):
        for g in range(hkv):
            hs = slice(g * G, (g + 1) * G)
            # shift: adding one vector to every key of the document changes nothing
            assert np.abs(dK[:, a:b, g].sum(axis=(0, 1))).max() < 1e-12
            # scale: (Q,K) -> (aQ, K/a) changes nothing
            lhs = (Q[:, a:b, hs] * dQ[:, a:b, hs]).sum()
            rhs = (K[:, a:b, g] * dK[:, a:b, g]).sum()
            assert abs(lhs - rhs) < 1e-11
            # mass: rows of P sum to one
            np.testing.assert_allclose(dV[:, a:b, g].sum(axis=(0, 1)), dO[:, a:b, hs].sum(axis=(0, 1, 2)),
                                       rtol=0, atol=1e-12)


# ---------------------------------------------------------------- independence properties
def test_independence_of_later_blocks_documents_and_step_ranges(oracle):
    k, cu, hq, hkv, d = 3, [0, 5, 11], 2, 2, 4
    Q, K, V, dO = rand_inputs(k, cu[-1], hq, hkv, d)
    scale = 0.5
    O, LSE, dQ, dK, dV = oracle.oracle_full(Q, K, V, cu, scale, dO)
    # later blocks do not influence earlier steps
    K2, V2 = K.copy(), V.copy()
    K2[2] += 3.0; V2[2] -= 1.0
    O2, *_ = oracle.oracle_full(Q, K2, V2, cu, scale)
    np.testing.assert_array_equal(O[:2], O2[:2])
    assert np.abs(O[2] - O2[2]).max() > 1e-3
    # a packed batch equals its documents run alone
    for a, b in zip(cu[:-1], cu[1:]):
        Oa, LSEa, dQa, dKa, dVa = oracle.oracle_full(Q[:, a:b], K[:, a:b], V[:, a:b], [0, b - a], scale, dO[:, a:b])
        np.testing.assert_allclose(O[:, a:b], Oa, rtol=0, atol=1e-15)
        np.testing.assert_allclose(dK[:, a:b], dKa, rtol=0, atol=1e-14)
        np.testing.assert_allclose(dQ[:, a:b], dQa, rtol=0, atol=1e-14)
    # step-at-a-time calls add up to the all-steps call
    dKs = np.zeros_like(dK); dVs = np.zeros_like(dV)
    for j in range(k):
        Oj, LSEj, dQj, dKj, dVj = oracle.oracle_full(Q, K, V, cu, scale, dO, j, j + 1)
        np.testing.assert_allclose(Oj[0], O[j], rtol=0, atol=1e-15)
        np.testing.assert_allclose(dQj[0], dQ[j], rtol=0, atol=1e-15)
        assert np.abs(dKj[j + 1:]).max(initial=0.0) == 0.0
        dKs += dKj; dVs += dVj
    np.testing.assert_allclose(dKs, dK, rtol=0, atol=1e-13)
    np.testing.assert_allclose(dVs, dV, rtol=0, atol=1e-13)


def test_f32_input_path_equals_f64_input_path(oracle):
    k, cu = 2, [0, 6, 9]
    Q, K, V, dO = rand_inputs(k, cu[-1], 2, 1, 4, dtype=np.float32)
    a = oracle.oracle_full(Q, K, V, cu, 0.5, dO)
    b = oracle.oracle_full(Q.astype(np.float64), K.astype(np.float64), V.astype(np.float64), cu, 0.5, dO.astype(np.float64))
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, rtol=0, atol=1e-13)   # same values; the compiler may order sums differently


def test_sampled_rows_equal_full_run_with_row_sparse_cotangent(oracle):
    k, cu, hq, hkv, d = 3, [0, 9, 14], 2, 1, 4
    Q, K, V, dO = rand_inputs(k, cu[-1], hq, hkv, d)
    rows = [(0, 0), (2, 8), (1, 9), (2, 13), (0, 5)]
    keep = np.zeros((k, cu[-1]), dtype=bool)
    for j, i in rows:
        keep[j, i] = True
    dOs = dO * keep[:, :, None, None]
    O, LSE, dQ, dK, dV = oracle.oracle_full(Q, K, V, cu, 0.5, dOs)
    rs = np.array([r[0] for r in rows], dtype=np.int32); rt = np.array([r[1] for r in rows], dtype=np.int32)
    r = oracle.oracle_run(Q, K, V, cu, 0.5, rs, rt, np.stack([dO[j, i] for j, i in rows]))
    for n, (j, i) in enumerate(rows):
        np.testing.assert_allclose(r.O[n], O[j, i], rtol=0, atol=1e-15)
        np.testing.assert_allclose(r.LSE[n], LSE[j, :, i], rtol=0, atol=1e-15)
        np.testing.assert_allclose(r.dQ[n], dQ[j, i], rtol=0, atol=1e-15)
    np.testing.assert_allclose(r.dK, dK, rtol=0, atol=1e-14)
    np.testing.assert_allclose(r.dV, dV, rtol=0, atol=1e-14)
