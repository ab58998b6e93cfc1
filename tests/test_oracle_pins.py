"""Pins for the fp64 oracle (CPU only).

Each test ties an oracle function to something other than itself: a value fixed by
the paper's definition and worked by hand, a closed form, a special case that
reduces to a library routine, brute force, or an independent restatement of the
operator.  Citations name the passage of the paper that fixes the expected value.
"""
import os

import numpy as np
import pytest

import oracle
from helpers import max_rel_err, parse_golden
from paper_2501_02573_amd import workloads as W

RNG = np.random.default_rng(1234)


def rand_qkv(B, H, N, d, rng=RNG):
    s = d ** -0.5
    return tuple(rng.standard_normal((B, H, N, d)) * s for _ in range(3))


# ---------------------------------------------------------------- hand-computed case
def test_hand_case_outputs_and_states(golden_dir):
    """Section 2.2 Eq. BCMV / Alg. 1 + App. C.1: N=3, d=2, gamma=0.5, worked by hand."""
    g = parse_golden(os.path.join(golden_dir, "hand_n3_d2.txt"))
    q, k, v = (g[n][None, None] for n in ("q", "k", "v"))
    gamma = g["gamma"].reshape(1)
    assert np.array_equal(oracle.quadratic(q, k, v, gamma)[0, 0], g["out"])
    out, s3 = oracle.recurrent(q, k, v, gamma)
    assert np.array_equal(out[0, 0], g["out"])
    assert np.array_equal(s3[0, 0], g["state3"])
    # token by token through decode_step: every intermediate state is fixed by the fixture
    S = np.zeros((1, 1, 2, 2))
    for i, name in enumerate(("state1", "state2", "state3")):
        o = oracle.decode_step(q[:, :, i], k[:, :, i], v[:, :, i], gamma, S)
        assert np.array_equal(S[0, 0], g[name])
        assert np.array_equal(o[0, 0], g["out"][i])
    # prefix runs give the same intermediate states
    for n, name in ((1, "state1"), (2, "state2")):
        _, s = oracle.recurrent(q[:, :, :n], k[:, :, :n], v[:, :, :n], gamma)
        assert np.array_equal(s[0, 0], g[name])
    for fn in (lambda: oracle.chunked(q, k, v, gamma, 2)[0], lambda: oracle.fleet(q, k, v, gamma),
               lambda: oracle.recursion(q, k, v, gamma, base=1)):
        assert np.allclose(fn()[0, 0], g["out"], rtol=0, atol=1e-14)


def test_toy_case_geometric_series(golden_dir):
    """App. C.1 toy case: q.k == 1 makes the operator the lambda-cumsum; v == 1 gives a geometric series."""
    g = parse_golden(os.path.join(golden_dir, "geometric_gamma_half.txt"))
    expect = g["out"].reshape(-1)
    N, d = expect.shape[0], 3
    q = np.zeros((1, 1, N, d)); k = np.zeros((1, 1, N, d))
    q[..., 0] = 1.0; k[..., 0] = 1.0               # q_i = k_j = e_1  =>  q_i . k_j = 1
    v = np.ones((1, 1, N, d))
    gamma = g["gamma"].reshape(1)
    for out in (oracle.quadratic(q, k, v, gamma), oracle.recurrent(q, k, v, gamma)[0]):
        assert np.array_equal(out[0, 0], np.repeat(expect[:, None], d, axis=1))
    i = np.arange(N)
    assert np.allclose(expect, (1 - 0.5 ** (i + 1)) / (1 - 0.5), rtol=0, atol=0)


def test_toy_case_is_discounted_cumsum():
    """App. C.1: with q_i . k_j = 1 the result is o_i = v_i + gamma o_{i-1} for arbitrary V."""
    N, d, g = 37, 5, 0.8125
    q = np.zeros((1, 1, N, d)); k = np.zeros((1, 1, N, d))
    q[..., 2] = 1.0; k[..., 2] = 1.0
    v = RNG.standard_normal((1, 1, N, d))
    ref = np.empty((N, d)); acc = np.zeros(d)
    for i in range(N):
        acc = v[0, 0, i] + g * acc
        ref[i] = acc
    assert np.allclose(oracle.quadratic(q, k, v, [g])[0, 0], ref, rtol=1e-14, atol=1e-14)
    assert np.allclose(oracle.recurrent(q, k, v, [g])[0][0, 0], ref, rtol=1e-14, atol=1e-14)


# ---------------------------------------------------------------- closed forms
def test_gamma_one_is_prefix_sum_attention():
    """Section 2.2: gamma = 1 is plain causal linear attention, o_i = q_i (sum_{j<=i} k_j^T v_j) (Eq. performer1/2)."""
    B, H, N, d = 2, 2, 50, 8
    q, k, v = rand_qkv(B, H, N, d)
    kv = np.einsum("bhne,bhnc->bhnec", k, v)
    U = np.cumsum(kv, axis=2)                       # library prefix sum
    ref = np.einsum("bhne,bhnec->bhnc", q, U)
    gamma = np.ones(H)
    assert max_rel_err(oracle.quadratic(q, k, v, gamma), ref) < 1e-13
    out, s = oracle.recurrent(q, k, v, gamma)
    assert max_rel_err(out, ref) < 1e-13
    assert np.allclose(s, U[:, :, -1], rtol=1e-13, atol=1e-13)
    # equals tril(QK^T) V computed with library matmuls
    ref2 = np.tril(q @ np.swapaxes(k, -1, -2)) @ v
    assert max_rel_err(oracle.quadratic(q, k, v, gamma), ref2) < 1e-13


def test_gamma_zero_keeps_only_the_diagonal():
    """M[i][i] = gamma^0 = 1 also for gamma = 0 (0^0 = 1): o_i = (q_i . k_i) v_i, state = k_N^T v_N."""
    B, H, N, d = 1, 3, 20, 4
    q, k, v = rand_qkv(B, H, N, d)
    ref = (q * k).sum(-1, keepdims=True) * v
    gamma = np.zeros(H)
    assert np.allclose(oracle.quadratic(q, k, v, gamma), ref, rtol=1e-14, atol=1e-15)
    out, s = oracle.recurrent(q, k, v, gamma)
    assert np.allclose(out, ref, rtol=1e-14, atol=1e-15)
    assert np.allclose(s, np.einsum("bhe,bhc->bhec", k[:, :, -1], v[:, :, -1]), rtol=1e-15, atol=0)
    assert np.allclose(oracle.chunked(q, k, v, gamma, 8)[0], ref, rtol=1e-14, atol=1e-15)


def test_single_token():
    """N = 1: o_0 = (q_0 . k_0) v_0 and the state is the outer product k_0^T v_0 (rows = key index)."""
    q, k, v = rand_qkv(2, 2, 1, 6)
    gamma = np.array([0.3, 0.95])
    ref = (q * k).sum(-1, keepdims=True) * v
    assert np.allclose(oracle.quadratic(q, k, v, gamma), ref, rtol=1e-15, atol=0)
    out, s = oracle.recurrent(q, k, v, gamma)
    assert np.allclose(out, ref, rtol=1e-15, atol=0)
    assert np.array_equal(s, k[:, :, 0, :, None] * v[:, :, 0, None, :])
    assert not np.allclose(s, np.swapaxes(s, -1, -2))   # the orientation is observable


def test_constant_kv_steady_state():
    """Recurrence of App. C.1 with fixed k, v: S_n = gamma^n S_0 + (1-gamma^n)/(1-gamma) k^T v -> k^T v/(1-gamma)."""
    d, g, n = 4, 0.75, 60
    k = RNG.standard_normal(d); v = RNG.standard_normal(d); q = RNG.standard_normal(d)
    S0 = RNG.standard_normal((d, d))
    S = S0.copy()[None, None]
    for _ in range(n):
        o = oracle.decode_step(q[None, None], k[None, None], v[None, None], [g], S)
    kv = np.outer(k, v)
    Sn = g ** n * S0 + (1 - g ** n) / (1 - g) * kv
    assert np.allclose(S[0, 0], Sn, rtol=1e-13, atol=1e-13)
    assert np.allclose(o[0, 0], q @ Sn, rtol=1e-13, atol=1e-13)
    assert np.allclose(S[0, 0], kv / (1 - g), rtol=1e-6, atol=1e-6)


def test_brute_force_scalar_loops():
    """Tiny case against a scalar triple loop written straight from Eq. BCMV with math.pow."""
    import math
    B, H, N, d = 1, 2, 7, 3
    q, k, v = rand_qkv(B, H, N, d)
    gamma = np.array([0.6, 0.0])
    ref = np.zeros((B, H, N, d))
    for b in range(B):
        for h in range(H):
            for i in range(N):
                for j in range(N):
                    if i >= j:
                        m = 1.0 if i == j else math.pow(gamma[h], i - j)
                        a = sum(q[b, h, i, e] * k[b, h, j, e] for e in range(d)) * m
                        for c in range(d):
                            ref[b, h, i, c] += a * v[b, h, j, c]
    assert np.allclose(oracle.quadratic(q, k, v, gamma), ref, rtol=1e-14, atol=1e-15)
    assert np.allclose(oracle.recurrent(q, k, v, gamma)[0], ref, rtol=1e-14, atol=1e-15)
    rows = np.array([[0, 6], [1, 0], [1, 3]])
    got = oracle.quadratic_rows(q, k, v, gamma, rows)
    assert np.allclose(got, np.stack([ref[0, 0, 6], ref[0, 1, 0], ref[0, 1, 3]]), rtol=1e-14, atol=1e-15)


# ---------------------------------------------------------------- structural properties
def test_linearity_and_shift():
    """O is linear in V and in Q; a leading token with k = v = 0 shifts every output down one row."""
    B, H, N, d = 1, 2, 33, 8
    q, k, v = rand_qkv(B, H, N, d)
    v2 = RNG.standard_normal(v.shape); q2 = RNG.standard_normal(q.shape)
    gamma = np.array([0.9, 0.5])
    f = lambda a, b_, c: oracle.recurrent(a, b_, c, gamma)[0]
    assert np.allclose(f(q, k, 2 * v + 3 * v2), 2 * f(q, k, v) + 3 * f(q, k, v2), rtol=1e-12, atol=1e-13)
    assert np.allclose(f(q - q2, k, v), f(q, k, v) - f(q2, k, v), rtol=1e-12, atol=1e-13)
    z = np.zeros((B, H, 1, d))
    qs, ks, vs = (np.concatenate([z if n else RNG.standard_normal(z.shape), x], axis=2)
                  for n, x in ((0, q), (1, k), (1, v)))
    shifted = oracle.quadratic(qs, ks, vs, gamma)
    assert np.allclose(shifted[:, :, 1:], oracle.quadratic(q, k, v, gamma), rtol=1e-13, atol=1e-14)
    assert np.all(shifted[:, :, 0] == 0)


def test_causality():
    """Row i depends on tokens j <= i only (M is lower triangular)."""
    q, k, v = rand_qkv(1, 1, 24, 4)
    base = oracle.quadratic(q, k, v, [0.9])
    k2, v2 = k.copy(), v.copy()
    k2[:, :, 10:] += 1.0; v2[:, :, 10:] -= 2.0
    pert = oracle.quadratic(q, k2, v2, [0.9])
    assert np.array_equal(base[:, :, :10], pert[:, :, :10])
    assert not np.allclose(base[:, :, 10:], pert[:, :, 10:])


def test_per_head_gamma_is_indexed_by_head_not_batch():
    B, H, N, d = 3, 2, 9, 4
    q, k, v = rand_qkv(B, H, N, d)
    gamma = np.array([0.2, 0.9])
    full = oracle.quadratic(q, k, v, gamma)
    for b in range(B):
        for h in range(H):
            one = oracle.quadratic(q[b:b + 1, h:h + 1], k[b:b + 1, h:h + 1], v[b:b + 1, h:h + 1], gamma[h:h + 1])
            assert np.array_equal(one[0, 0], full[b, h])
    rec = oracle.recurrent(q, k, v, gamma)[0]
    assert max_rel_err(rec, full) < 1e-13


# ---------------------------------------------------------------- independent forms agree
@pytest.mark.parametrize("cfg", [W.CONFIG1, W.CONFIG2], ids=lambda c: c.name)
def test_two_forms_agree_on_benchmark_configs(cfg):
    """Form 1 (Eq. BCMV) and form 2 (Alg. 1 + App. C.1) agree to 1e-12 on the seeded workloads."""
    q, k, v, gamma = W.make_forward_inputs(cfg)
    q, k, v, gamma = (W.to_f64(t) for t in (q, k, v, gamma))
    a = oracle.quadratic(q, k, v, gamma)
    b, _ = oracle.recurrent(q, k, v, gamma)
    assert max_rel_err(b, a) < 1e-12


def test_two_forms_agree_bf16_inputs_sampled_rows():
    """Same agreement at d=128 with bf16-rounded inputs and long memory, on sampled rows of form 1."""
    q, k, v, gamma = W.make_custom_forward_inputs(1, 4, 3000, 128, "bf16", 7, W.make_gamma("pow2:5:10", 4))
    q, k, v, gamma = (W.to_f64(t) for t in (q, k, v, gamma))
    rec, _ = oracle.recurrent(q, k, v, gamma)
    rows = np.array([[bh, i] for bh in range(4) for i in (0, 1, 63, 64, 65, 1000, 2047, 2999)])
    got = oracle.quadratic_rows(q, k, v, gamma, rows)
    ref = np.stack([rec.reshape(4, 3000, 128)[bh, i] for bh, i in rows])
    assert np.abs(got - ref).max() / np.abs(ref).max() < 1e-12


@pytest.mark.parametrize("chunk", [1, 16, 64, 128, 200, 333])
def test_chunk_size_invariance(chunk):
    """Alg. 2 with the decay split of Alg. 4: any block size, ragged tail included, gives the same O and state."""
    B, H, N, d = 1, 3, 333, 16
    q, k, v = rand_qkv(B, H, N, d)
    gamma = np.array([1.0, 0.97, 0.5])
    ref, s_ref = oracle.recurrent(q, k, v, gamma)
    out, s = oracle.chunked(q, k, v, gamma, chunk)
    assert max_rel_err(out, ref) < 1e-12
    assert max_rel_err(s, s_ref) < 1e-12
    assert max_rel_err(out, oracle.quadratic(q, k, v, gamma)) < 1e-12


def test_fleet_and_recursion_identities():
    """Eq. p with the lambda-cumsum (App. C.1) and Alg. 4 reproduce Eq. BCMV."""
    B, H, N, d = 1, 2, 45, 6
    q, k, v = rand_qkv(B, H, N, d)
    gamma = np.array([0.85, 1.0])
    ref = oracle.quadratic(q, k, v, gamma)
    assert max_rel_err(oracle.fleet(q, k, v, gamma), ref) < 1e-12
    for base in (1, 4, 32):
        assert max_rel_err(oracle.recursion(q, k, v, gamma, base=base), ref) < 1e-12


def test_fleet_identity_with_rank_different_from_width():
    """Eq. p for B, C of width r and V of width d != r (Section 2.2) against Eq. BCMV written out."""
    rng = np.random.default_rng(17)
    Bn, H, N, r, d = 1, 2, 23, 5, 9
    q, k = rng.standard_normal((Bn, H, N, r)), rng.standard_normal((Bn, H, N, r))
    v = rng.standard_normal((Bn, H, N, d))
    gamma = np.array([0.7, 1.0])
    ref = np.zeros_like(v)
    for h in range(H):
        for i in range(N):
            for j in range(i + 1):
                ref[0, h, i] += gamma[h] ** (i - j) * (q[0, h, i] @ k[0, h, j]) * v[0, h, j]
    assert max_rel_err(oracle.fleet(q, k, v, gamma), ref) < 1e-12
    assert max_rel_err(oracle.quadratic(q, k, v, gamma), ref) < 1e-12


def test_state_carry_prefill_then_decode():
    """Splitting a sequence: recurrent(first part) -> state -> recurrent/decode(rest) equals one pass."""
    B, H, N, d = 2, 2, 40, 8
    q, k, v = rand_qkv(B, H, N, d)
    gamma = np.array([0.9, 0.99])
    full, s_full = oracle.recurrent(q, k, v, gamma)
    n0 = 17
    o0, s0 = oracle.recurrent(q[:, :, :n0], k[:, :, :n0], v[:, :, :n0], gamma)
    o1, s1 = oracle.recurrent(q[:, :, n0:], k[:, :, n0:], v[:, :, n0:], gamma, state_in=s0)
    assert np.allclose(np.concatenate([o0, o1], axis=2), full, rtol=1e-13, atol=1e-14)
    assert np.allclose(s1, s_full, rtol=1e-13, atol=1e-14)
    S = s0.copy()
    for i in range(n0, N):
        o = oracle.decode_step(q[:, :, i], k[:, :, i], v[:, :, i], gamma, S)
        assert np.allclose(o, full[:, :, i], rtol=1e-13, atol=1e-14)
    assert np.allclose(S, s_full, rtol=1e-13, atol=1e-14)
    oc, sc = oracle.chunked(q[:, :, n0:], k[:, :, n0:], v[:, :, n0:], gamma, 8, state_in=s0)
    assert np.allclose(oc, full[:, :, n0:], rtol=1e-12, atol=1e-13)
    assert np.allclose(sc, s_full, rtol=1e-12, atol=1e-13)


def test_empty_sequence_leaves_the_state_as_it_entered():
    """N = 0: the loops of Alg. 1 and Alg. 2 do not run.  No output rows; the state is handed on
    unchanged (zero without an entering state); and a sequence split as [] + [all] or [all] + []
    gives what one pass gives."""
    B, H, N, d = 2, 3, 11, 8
    q, k, v = rand_qkv(B, H, N, d)
    gamma = np.array([0.9, 0.5, 1.0])
    s_in = np.random.default_rng(5).standard_normal((B, H, d, d))
    e = np.zeros((B, H, 0, d))
    o, s = oracle.recurrent(e, e, e, gamma, state_in=s_in)
    assert o.shape == (B, H, 0, d) and np.array_equal(s, s_in)
    o, s = oracle.recurrent(e, e, e, gamma)
    assert o.shape == (B, H, 0, d) and np.array_equal(s, np.zeros((B, H, d, d)))
    assert oracle.quadratic(e, e, e, gamma).shape == (B, H, 0, d)
    assert oracle.fleet(e, e, e, gamma).shape == (B, H, 0, d)
    oc, sc = oracle.chunked(e, e, e, gamma, 4, state_in=s_in)
    assert oc.shape == (B, H, 0, d) and np.array_equal(sc, s_in)
    full, s_full = oracle.recurrent(q, k, v, gamma, state_in=s_in)
    _, s0 = oracle.recurrent(e, e, e, gamma, state_in=s_in)
    o1, s1 = oracle.recurrent(q, k, v, gamma, state_in=s0)
    assert np.array_equal(o1, full) and np.array_equal(s1, s_full)
    _, s2 = oracle.recurrent(e, e, e, gamma, state_in=s_full)
    assert np.array_equal(s2, s_full)
    with pytest.raises(Exception):
        oracle.recurrent(np.zeros((B, H, 3, d)), np.zeros((B, H, 3, d)), np.zeros((B, H, 2, d)), gamma)


# ---------------------------------------------------------------- planted mistakes are caught
def _mutants():
    """Plausible wrong versions of form 2, written here (numpy), to show the pins above would fail on them."""
    def run(q, k, v, g, update, output_before=False):
        N, d = q.shape
        S = np.zeros((d, d)); out = np.zeros((N, d))
        for i in range(N):
            if output_before:
                out[i] = q[i] @ S
            S = update(S, k[i], v[i], g)
            if not output_before:
                out[i] = q[i] @ S
        return out
    good = lambda S, k, v, g: g * S + np.outer(k, v)
    return {
        "correct": lambda q, k, v, g: run(q, k, v, g, good),
        "exclusive_diagonal": lambda q, k, v, g: run(q, k, v, g, good, output_before=True),
        "no_decay": lambda q, k, v, g: run(q, k, v, g, lambda S, k, v, g_: S + np.outer(k, v)),
        "transposed_state": lambda q, k, v, g: run(q, k, v, g, lambda S, k, v, g_: g_ * S + np.outer(v, k)),
        "decay_applied_to_new_term": lambda q, k, v, g: run(q, k, v, g, lambda S, k, v, g_: g_ * (S + np.outer(k, v))),
        "sign": lambda q, k, v, g: run(q, k, v, g, lambda S, k, v, g_: g_ * S - np.outer(k, v)),
    }


def test_hand_case_rejects_planted_mistakes(golden_dir):
    g = parse_golden(os.path.join(golden_dir, "hand_n3_d2.txt"))
    m = _mutants()
    assert np.array_equal(m["correct"](g["q"], g["k"], g["v"], 0.5), g["out"])
    for name, fn in m.items():
        if name != "correct":
            assert not np.allclose(fn(g["q"], g["k"], g["v"], 0.5), g["out"]), name


# ---------------------------------------------------------------- rank r different from the value width dv (Section 2.2)
def _rand_rd(B, H, N, r, dv, seed):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, H, N, r))
    k = rng.standard_normal((B, H, N, r))
    v = rng.standard_normal((B, H, N, dv))
    gamma = rng.uniform(0.3, 1.0, size=H)
    return q, k, v, gamma


@pytest.mark.parametrize("r,dv", [(3, 5), (5, 3), (4, 8)])
def test_rank_differs_from_value_width(r, dv):
    """B, C in R^(N x r), V in R^(N x d): pinned by library matmuls, by zero padding to the square
    case (which the other pins hold down), and by agreement of the two forms."""
    B, H, N = 2, 3, 37
    q, k, v, gamma = _rand_rd(B, H, N, r, dv, seed=r * 10 + dv)
    quad = oracle.quadratic(q, k, v, gamma)
    rec, s_out = oracle.recurrent(q, k, v, gamma)
    assert quad.shape == (B, H, N, dv) and s_out.shape == (B, H, r, dv)
    # the definition by numpy routines: tril of (Q K^T) .* M, then @ V
    i = np.arange(N)
    for h in range(H):
        M = np.tril(gamma[h] ** np.clip(i[:, None] - i[None, :], 0, None))
        ref = np.matmul(np.matmul(q[:, h], np.swapaxes(k[:, h], 1, 2)) * M, v[:, h])
        np.testing.assert_allclose(quad[:, h], ref, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(rec, quad, rtol=1e-11, atol=1e-12)
    # final state = sum_j gamma^(N-1-j) k_j^T v_j
    for h in range(H):
        wts = gamma[h] ** (N - 1 - i)
        ref_s = np.einsum("j,bjr,bjc->brc", wts, k[:, h], v[:, h])
        np.testing.assert_allclose(s_out[:, h], ref_s, rtol=1e-11, atol=1e-12)
    # zero padding to a square problem changes nothing
    d = max(r, dv)
    qp = np.zeros((B, H, N, d)); kp = np.zeros((B, H, N, d)); vp = np.zeros((B, H, N, d))
    qp[..., :r] = q; kp[..., :r] = k; vp[..., :dv] = v
    sq = oracle.quadratic(qp, kp, vp, gamma)
    np.testing.assert_allclose(sq[..., :dv], quad, rtol=1e-13, atol=1e-13)
    assert np.all(sq[..., dv:] == 0.0)
    # the recurrence carries across a split, and a decode step continues it
    n0 = 20
    o1, s1 = oracle.recurrent(q[:, :, :n0], k[:, :, :n0], v[:, :, :n0], gamma)
    o2, s2 = oracle.recurrent(q[:, :, n0:N - 1], k[:, :, n0:N - 1], v[:, :, n0:N - 1], gamma, state_in=s1)
    s2 = np.ascontiguousarray(s2)
    o3 = oracle.decode_step(q[:, :, N - 1], k[:, :, N - 1], v[:, :, N - 1], gamma, s2)
    np.testing.assert_allclose(np.concatenate([o1, o2, o3[:, :, None]], axis=2), rec, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(s2, s_out, rtol=1e-11, atol=1e-12)
