"""TEST INFRASTRUCTURE ONLY: dense-concatenated form of TTT attention in numpy fp64.

The k steps are laid side by side as one sequence of k*Q_LEN slots and attention is ordinary masked
attention over it: the explicit boolean mask is Alg. 2's predicate evaluated on flat indices, every
score is computed and masked ones are set to -inf, softmax in fp64.  For small inputs; it is the
second, independently written form that the row-mask oracle in ttt_oracle.c is compared with.
"""
from __future__ import annotations

import numpy as np


def dense_mask_alg2(k: int, q_len: int, seq_len: int, step: int) -> np.ndarray:
    """Alg. 2 as printed, for ONE padded sequence: queries q_i in [0,Q_LEN) of TTT step `step`,
    key/value slots kv_i in [0,(step+1)*Q_LEN) (the cache holds step+1 blocks, Sec. 4.2.1), the
    remaining slots up to k*Q_LEN are not in the cache yet and stay False.

    Returns bool [Q_LEN, k*Q_LEN]."""
    q_i = np.arange(q_len)[:, None]
    kv_i = np.arange(k * q_len)[None, :]
    m_causal = q_i >= kv_i
    m_pad = kv_i < seq_len
    M_causal = m_causal & m_pad
    m_suffix = kv_i >= q_len
    m_pad2 = (kv_i % q_len) < seq_len
    m_diag = ((kv_i - q_i) % q_len) == 0
    M_suffix = m_suffix & m_pad2 & m_diag
    M = M_causal | M_suffix
    M = M & (kv_i < (step + 1) * q_len)
    return M


def packed_mask(k: int, cu_seqlens) -> np.ndarray:
    """Mask [k*T, k*T] for a packed batch: each document is one padded sequence of Alg. 2 with
    Q_LEN = T_alg2 = its own length (no pad rows), and documents never see each other."""
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    T = int(cu[-1])
    M = np.zeros((k * T, k * T), dtype=bool)
    for r in range(len(cu) - 1):
        a, b = int(cu[r]), int(cu[r + 1])
        L = b - a
        if L == 0:
            continue
        for j in range(k):
            Md = dense_mask_alg2(k, L, L, j)            # [L, k*L]
            for l in range(k):
                M[j * T + a:j * T + b, l * T + a:l * T + b] = Md[:, l * L:(l + 1) * L]
    return M


def dense_forward_backward(Q, K, V, cu_seqlens, scale, dO=None):
    """Q [k,T,hq,d], K,V [k,T,hkv,d] float64.  Returns O [k,T,hq,d], LSE [k,hq,T] and, with dO,
    dQ, dK, dV -- all steps, dense formulas on the concatenated sequence."""
    Q = np.asarray(Q, dtype=np.float64); K = np.asarray(K, dtype=np.float64); V = np.asarray(V, dtype=np.float64)
    k, T, hq, d = Q.shape
    hkv = K.shape[2]
    G = hq // hkv
    M = packed_mask(k, cu_seqlens)
    n = k * T
    O = np.zeros((k, T, hq, d)); LSE = np.zeros((k, hq, T))
    dQ = dK = dV = None
    if dO is not None:
        dO = np.asarray(dO, dtype=np.float64)
        dQ = np.zeros_like(Q); dK = np.zeros_like(K); dV = np.zeros_like(V)
    for h in range(hq):
        g = h // G
        Qc = Q[:, :, h, :].reshape(n, d)
        Kc = K[:, :, g, :].reshape(n, d)
        Vc = V[:, :, g, :].reshape(n, d)
        S = scale * (Qc @ Kc.T)
        S = np.where(M, S, -np.inf)
        mx = S.max(axis=1, keepdims=True)
        E = np.exp(S - mx)
        Z = E.sum(axis=1, keepdims=True)
        P = E / Z
        Oc = P @ Vc
        O[:, :, h, :] = Oc.reshape(k, T, d)
        LSE[:, h, :] = (mx + np.log(Z)).reshape(k, T)
        if dO is not None:
            dOc = dO[:, :, h, :].reshape(n, d)
            dVc = P.T @ dOc
            dP = dOc @ Vc.T
            Dd = (dOc * Oc).sum(axis=1, keepdims=True)
            dS = P * (dP - Dd)
            dQ[:, :, h, :] = (scale * (dS @ Kc)).reshape(k, T, d)
            dK[:, :, g, :] += (scale * (dS.T @ Qc)).reshape(k, T, d)
            dV[:, :, g, :] += dVc.reshape(k, T, d)
    return O, LSE, dQ, dK, dV
