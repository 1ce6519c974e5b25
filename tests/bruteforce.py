"""Independent numpy fp64 definitions used to pin the oracle (no code shared with it).

Token-level, dense, O(N^2): the textbook operators the block-level SLA must reduce to.
"""
from __future__ import annotations

import numpy as np


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def dense_attention(Q, K, V, scale):
    """Softmax(Q K^T * scale) V for one head, fp64 (the paper's A_full, section 3.3)."""
    S = Q @ K.T * scale
    S = S - S.max(axis=1, keepdims=True)
    P = np.exp(S)
    return (P / P.sum(axis=1, keepdims=True)) @ V


def phi_softmax(X):
    E = np.exp(X - X.max(axis=-1, keepdims=True))
    return E / E.sum(axis=-1, keepdims=True)


def phi_elu1(X):
    """ELU(x) + 1 as Alg. 1 step 6 prints it: x + 1 where x > 0, exp(x) elsewhere."""
    return np.where(X > 0, X + 1.0, np.exp(np.minimum(X, 0.0)))


PHI = {"softmax": phi_softmax, "elu1": phi_elu1}


def linear_attention(Q, K, V, W, phi="softmax"):
    """Alg. 1 steps 6-10 with O_sparse = 0, one head."""
    fq, fk = PHI[phi](Q), PHI[phi](K)
    T = fk.T @ V                      # [D, D]
    z = fk.sum(axis=0)                # [D]
    return ((fq @ T) / (fq @ z)[:, None]) @ W


def rank_labels(s_row, k_c, k_n):
    """Definition of the three-way labels by explicit rank counting (O(n^2))."""
    n = len(s_row)
    lab = np.empty(n, dtype=np.int8)
    for j in range(n):
        r = sum(1 for jj in range(n) if s_row[jj] > s_row[j] or (s_row[jj] == s_row[j] and jj < j))
        lab[j] = 2 if r < k_c else (0 if r >= n - k_n else 1)
    return lab


def sla_tokenlevel(Q, K, V, W, labels_row_of_block, bq, bk, scale, phi="softmax"):
    """SLA for one head from given labels [Nqb, Nkb], written with dense token masks."""
    N = Q.shape[0]
    qb = np.arange(N) // bq
    kb = np.arange(N) // bk
    L = labels_row_of_block[qb][:, kb]          # [N, N] label of (query token, key token)
    S = Q @ K.T * scale
    out = np.zeros_like(V)
    crit = L == 2
    Sm = np.where(crit, S, -np.inf)
    has = crit.any(axis=1)
    m = np.where(has, Sm.max(axis=1, initial=-np.inf), 0.0)
    P = np.where(crit, np.exp(Sm - m[:, None]), 0.0)
    den = P.sum(axis=1)
    out[has] = (P[has] / den[has, None]) @ V
    fq, fk = PHI[phi](Q), PHI[phi](K)
    A = np.where(L == 1, fq @ fk.T, 0.0)        # phi(q).phi(k) on marginal pairs
    dl = A.sum(axis=1)
    hasm = (L == 1).any(axis=1)
    lin = np.zeros_like(V)
    lin[hasm] = (A[hasm] @ V) / dl[hasm, None]
    return out + lin @ W, out, lin
