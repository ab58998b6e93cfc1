"""Randomised properties of the fp64 oracle (CPU only), complementing the fixed pins.

Each property follows from the definition O = ((Q K^T) .* M) V, M[i][j] = gamma^(i-j) for i >= j
(Section 2.2, Eq. "BCMV"), not from any implementation: two forms agree; outputs do not depend on
later tokens; the operator is linear in V and in Q; a split sequence carries through its state;
scaling the decay of a key by hand reproduces a shifted problem.
"""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle

shapes = st.tuples(st.integers(1, 2), st.integers(1, 3), st.integers(1, 70), st.integers(1, 9), st.integers(1, 9))
gammas = st.sampled_from([0.0, 0.3, 0.9, 0.999, 1.0])


def draw(shape, seed, g):
    B, H, N, r, dv = shape
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, H, N, r))
    k = rng.standard_normal((B, H, N, r))
    v = rng.standard_normal((B, H, N, dv))
    gamma = np.full(H, g)
    if H > 1:
        gamma[1:] = rng.uniform(0.0, 1.0, size=H - 1)
    return q, k, v, gamma


@settings(max_examples=40, deadline=None)
@given(shapes, st.integers(0, 10 ** 6), gammas)
def test_forms_agree_and_are_causal(shape, seed, g):
    q, k, v, gamma = draw(shape, seed, g)
    quad = oracle.quadratic(q, k, v, gamma)
    rec, _ = oracle.recurrent(q, k, v, gamma)
    scale = max(np.abs(quad).max(), 1e-300)
    assert np.abs(quad - rec).max() <= 1e-12 * scale
    # causality: perturbing tokens >= m leaves outputs < m untouched (bitwise, same arithmetic)
    N = shape[2]
    m = seed % N
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    q2[:, :, m:] += 1.0; k2[:, :, m:] -= 2.0; v2[:, :, m:] *= 3.0
    assert np.array_equal(oracle.quadratic(q2, k2, v2, gamma)[:, :, :m], quad[:, :, :m])
    assert np.array_equal(oracle.recurrent(q2, k2, v2, gamma)[0][:, :, :m], rec[:, :, :m])


@settings(max_examples=30, deadline=None)
@given(shapes, st.integers(0, 10 ** 6), gammas)
def test_linearity_and_state_carry(shape, seed, g):
    q, k, v, gamma = draw(shape, seed, g)
    rng = np.random.default_rng(seed + 1)
    v_b = rng.standard_normal(v.shape)
    a, b = 0.75, -1.5
    lhs, _ = oracle.recurrent(q, k, a * v + b * v_b, gamma)
    o1, _ = oracle.recurrent(q, k, v, gamma)
    o2, _ = oracle.recurrent(q, k, v_b, gamma)
    scale = max(np.abs(o1).max(), np.abs(o2).max(), 1e-300)
    assert np.abs(lhs - (a * o1 + b * o2)).max() <= 1e-11 * scale
    # split anywhere: the state carries the past exactly (same additions in the same order)
    N = shape[2]
    m = seed % (N + 1)
    if 0 < m < N:
        oa, sa = oracle.recurrent(q[:, :, :m], k[:, :, :m], v[:, :, :m], gamma)
        ob, sb = oracle.recurrent(q[:, :, m:], k[:, :, m:], v[:, :, m:], gamma, state_in=sa)
        full, sf = oracle.recurrent(q, k, v, gamma)
        assert np.array_equal(np.concatenate([oa, ob], axis=2), full)
        assert np.array_equal(sb, sf)


@settings(max_examples=25, deadline=None)
@given(st.integers(2, 60), st.integers(1, 6), st.integers(0, 10 ** 6), st.sampled_from([0.5, 0.9, 1.0]))
def test_chunked_form_matches_for_any_chunk_size(N, d, seed, g):
    rng = np.random.default_rng(seed)
    q, k, v = (rng.standard_normal((1, 2, N, d)) for _ in range(3))
    gamma = np.array([g, rng.uniform(0.1, 1.0)])
    ref, s_ref = oracle.recurrent(q, k, v, gamma)
    chunk = 1 + seed % N
    out, s_out = oracle.chunked(q, k, v, gamma, chunk)
    scale = max(np.abs(ref).max(), 1e-300)
    assert np.abs(out - ref).max() <= 1e-11 * scale
    assert np.abs(s_out - s_ref).max() <= 1e-11 * max(np.abs(s_ref).max(), 1e-300)
