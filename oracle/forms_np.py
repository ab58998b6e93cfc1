"""Further fp64 forms of the same operator, in numpy -- TEST INFRASTRUCTURE ONLY.

These restate, each in its own way, what the C oracle computes; the tests play
them against one another and against closed forms.

``chunked``    the block-based algorithm (Appendix B.2, Alg. 2) carried over to
               the decaying mask.  The paper prints the block equations for the
               0/1 mask only; the decayed version follows from the partition
               identity of Section 3.3 and the W1/W2 weight split of the
               recursion with a special mask (Appendix B.3, Alg. 4):
                   O_t     = ((Q_t K_t^T) .* D) V_t + Lam Q_t S_t
                   S_{t+1} = gamma^L S_t + (Gam K_t)^T V_t
               with L the block length, D[i][j] = gamma^(i-j) (i >= j),
               Lam = diag(gamma^1..gamma^L), Gam = diag(gamma^(L-1)..gamma^0).
               The inter-block sum runs over earlier blocks only (the printed
               sum's upper limit i would count block i twice; Alg. 2 itself
               uses U before updating it).
``fleet``      FleetAttention (Section 3.1, Eq. "p") with the lambda-cumsum of
               Appendix C.1: O = sum_r diag(b_r) lambda-cumsum(diag(c_r) V).
``recursion``  the recursive split with the decaying mask (Appendix B.3, Alg. 4).
"""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np


def _as4(q, k, v, gamma):
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    gamma = np.asarray(gamma, dtype=np.float64).reshape(-1)
    assert q.ndim == 4 and q.shape == k.shape == v.shape and gamma.shape[0] == q.shape[1]
    return q, k, v, gamma


def _decay_mask(g: float, n: int) -> np.ndarray:
    """n x n matrix with gamma^(i-j) on and below the diagonal (0^0 = 1), 0 above."""
    idx = np.arange(n)
    diff = idx[:, None] - idx[None, :]
    m = np.power(g, np.maximum(diff, 0).astype(np.float64))
    return np.where(diff >= 0, m, 0.0)


def chunked(q, k, v, gamma, chunk: int, state_in: Optional[np.ndarray] = None
            ) -> Tuple[np.ndarray, np.ndarray]:
    """Block algorithm with decay; returns (out, final state).  ``chunk`` need not divide N."""
    q, k, v, gamma = _as4(q, k, v, gamma)
    B, H, N, d = q.shape
    out = np.zeros_like(q)
    s_out = np.zeros((B, H, d, d))
    for b in range(B):
        for h in range(H):
            g = float(gamma[h])
            S = np.zeros((d, d)) if state_in is None else np.array(state_in[b, h], dtype=np.float64)
            for t0 in range(0, N, chunk):
                L = min(chunk, N - t0)
                Q, K, V = q[b, h, t0:t0 + L], k[b, h, t0:t0 + L], v[b, h, t0:t0 + L]
                lam = np.power(g, np.arange(1, L + 1, dtype=np.float64))          # gamma^(i+1), i = 0..L-1
                gam = np.power(g, np.arange(L - 1, -1, -1, dtype=np.float64))     # gamma^(L-1-j)
                intra = ((Q @ K.T) * _decay_mask(g, L)) @ V
                inter = lam[:, None] * (Q @ S)
                out[b, h, t0:t0 + L] = intra + inter
                S = np.power(g, float(L)) * S + (gam[:, None] * K).T @ V
            s_out[b, h] = S
    return out, s_out


def _lambda_cumsum(x: np.ndarray, lam: float) -> np.ndarray:
    """y_i = x_i + lam * y_{i-1} along axis 0 (Appendix C.1)."""
    y = np.empty_like(x)
    acc = np.zeros(x.shape[1:], dtype=x.dtype)
    for i in range(x.shape[0]):
        acc = x[i] + lam * acc
        y[i] = acc
    return y


def fleet(q, k, v, gamma) -> np.ndarray:
    """Rank-by-rank form: sum over columns r of Q, K of diag(q_r) lambda-cumsum(diag(k_r) V).

    Q and K are N x r, V is N x d (Section 2.2): the rank need not equal the value width."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    gamma = np.asarray(gamma, dtype=np.float64).reshape(-1)
    assert q.ndim == 4 and q.shape == k.shape and v.shape[:3] == q.shape[:3] and gamma.shape[0] == q.shape[1]
    B, H, N, d = q.shape
    out = np.zeros_like(v)
    for b in range(B):
        for h in range(H):
            for r in range(d):
                out[b, h] += q[b, h, :, r:r + 1] * _lambda_cumsum(k[b, h, :, r:r + 1] * v[b, h], float(gamma[h]))
    return out


def _recursion_2d(Bm, Cm, Vm, w: float, base: int) -> np.ndarray:
    n = Bm.shape[0]
    if n <= base:
        return ((Bm @ Cm.T) * _decay_mask(w, n)) @ Vm
    mid = n // 2
    o1 = _recursion_2d(Bm[:mid], Cm[:mid], Vm[:mid], w, base)
    o2 = _recursion_2d(Bm[mid:], Cm[mid:], Vm[mid:], w, base)
    w1 = np.power(w, np.arange(0, n - mid, dtype=np.float64))        # 1, w, ..., w^(right-mid-1)
    w2 = np.power(w, np.arange(mid, 0, -1, dtype=np.float64))        # w^(mid-left), ..., w
    o3 = (w1[:, None] * Bm[mid:]) @ ((w2[:, None] * Cm[:mid]).T @ Vm[:mid])
    return np.concatenate([o1, o2 + o3], axis=0)


def recursion(q, k, v, gamma, base: int = 4) -> np.ndarray:
    """Recursive halves with the W1/W2 decay split (Alg. 4); ``base`` = termination block size."""
    q, k, v, gamma = _as4(q, k, v, gamma)
    B, H, N, d = q.shape
    out = np.empty_like(v)
    for b in range(B):
        for h in range(H):
            out[b, h] = _recursion_2d(q[b, h], k[b, h], v[b, h], float(gamma[h]), base)
    return out
