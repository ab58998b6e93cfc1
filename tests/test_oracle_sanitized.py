"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

``oracle/leet_oracle.c`` is compiled together with ``oracle/sanitize_driver.c`` into a standalone
program with ``-fsanitize=address,undefined`` (the runtimes linked statically, so nothing has to be
preloaded), run on cases whose buffers are allocated at their exact sizes, and what it computes is
held against the same pins as the regular build: the hand-worked case of ``tests/golden``, closed
forms, and the regular build's results.  A sanitizer report makes the program exit non-zero."""
import os
import subprocess

import numpy as np
import pytest

import oracle
from helpers import parse_golden

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san") / "oracle_sanitized")
    cmd = ["gcc", "-std=c99", "-O1", "-g", "-fopenmp", "-fno-omit-frame-pointer",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
           "-Wall", "-Wextra", "-o", exe,
           os.path.join(ROOT, "oracle", "sanitize_driver.c"), os.path.join(ROOT, "oracle", "leet_oracle.c"), "-lm"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    return exe


def run_case(driver, tmp_path, q, k, v, gamma, state_in=None, rows=None):
    q, k, v = (np.ascontiguousarray(a, dtype=np.float64) for a in (q, k, v))
    gamma = np.ascontiguousarray(gamma, dtype=np.float64).reshape(-1)
    B, H, N, r = q.shape
    dv = v.shape[3]
    rows = np.zeros((0, 2), dtype=np.int64) if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    case, result = str(tmp_path / "case.bin"), str(tmp_path / "result.bin")
    with open(case, "wb") as f:
        np.array([B, H, N, r, dv, int(state_in is not None), len(rows)], dtype=np.int64).tofile(f)
        for a in (q, k, v, gamma):
            a.tofile(f)
        if state_in is not None:
            np.ascontiguousarray(state_in, dtype=np.float64).tofile(f)
        rows.tofile(f)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    res = subprocess.run([driver, case, result], capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0, f"sanitized oracle failed (rc {res.returncode}):\n{res.stderr[-4000:]}"
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr[-4000:]
    flat = np.fromfile(result, dtype=np.float64)
    sizes = [B * H * N * dv, B * H * N * dv, B * H * r * dv, len(rows) * dv, B * H * dv, B * H * r * dv]
    assert flat.size == sum(sizes)
    parts = np.split(flat, np.cumsum(sizes)[:-1])
    return {"quadratic": parts[0].reshape(B, H, N, dv), "recurrent": parts[1].reshape(B, H, N, dv),
            "state_out": parts[2].reshape(B, H, r, dv), "quadratic_rows": parts[3].reshape(len(rows), dv),
            "decode_out": parts[4].reshape(B, H, dv), "decode_state": parts[5].reshape(B, H, r, dv)}


def test_hand_case_under_sanitizers(driver, tmp_path, golden_dir):
    """The hand-worked N = 3, d = 2, gamma = 0.5 case (Eq. "BCMV" and Alg. 1 by hand): outputs and final state."""
    g = parse_golden(os.path.join(golden_dir, "hand_n3_d2.txt"))
    q, k, v = (g[n].reshape(1, 1, 3, 2) for n in ("q", "k", "v"))
    got = run_case(driver, tmp_path, q, k, v, [0.5], rows=[[0, 0], [0, 2]])
    np.testing.assert_allclose(got["quadratic"][0, 0], g["out"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(got["recurrent"][0, 0], g["out"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(got["state_out"][0, 0], g["state3"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(got["quadratic_rows"], g["out"][[0, 2]], rtol=0, atol=1e-14)
    np.testing.assert_allclose(got["decode_state"][0, 0], g["state1"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(got["decode_out"][0, 0], g["out"][0], rtol=0, atol=1e-14)


CASES = [
    # B, H, N, r, dv, with_state: ragged sizes, one token, rank different from the value width
    (1, 1, 1, 2, 2, False), (2, 3, 37, 8, 8, True), (1, 2, 65, 16, 16, False), (1, 3, 20, 3, 5, True),
    (2, 1, 9, 5, 3, False), (1, 4, 130, 4, 8, True),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "B%d_H%d_N%d_r%d_dv%d_s%d" % c)
def test_sanitized_build_agrees_with_the_pins(driver, tmp_path, case):
    B, H, N, r, dv, with_state = case
    rng = np.random.default_rng(N * 31 + r)
    q, k = rng.standard_normal((2, B, H, N, r))
    v = rng.standard_normal((B, H, N, dv))
    gamma = np.array(([0.0, 1.0, 0.5, 0.97] * 2)[:H])
    s_in = rng.standard_normal((B, H, r, dv)) if with_state else None
    rows = np.array([[bh, i] for bh in range(B * H) for i in sorted({0, N - 1, N // 2})]) if r == dv else None
    got = run_case(driver, tmp_path, q, k, v, gamma, s_in, rows)
    # the regular build on the same inputs
    ref_rec, ref_state = oracle.recurrent(q, k, v, gamma, state_in=s_in)
    np.testing.assert_allclose(got["recurrent"], ref_rec, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(got["state_out"], ref_state, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(got["quadratic"], oracle.quadratic(q, k, v, gamma), rtol=1e-13, atol=1e-13)
    # the definition by library routines: tril(Q K^T .* gamma^(i-j)) V  (+ the entering state's share)
    i, j = np.arange(N)[:, None], np.arange(N)[None, :]
    for b in range(B):
        for h in range(H):
            with np.errstate(divide="ignore"):
                M = np.where(i >= j, np.power(gamma[h], np.maximum(i - j, 0).astype(float)), 0.0)
            want = ((q[b, h] @ k[b, h].T) * M) @ v[b, h]
            np.testing.assert_allclose(got["quadratic"][b, h], want, rtol=1e-11, atol=1e-11)
            if with_state:
                want = want + (np.power(gamma[h], np.arange(1, N + 1, dtype=float))[:, None] * q[b, h]) @ s_in[b, h]
            np.testing.assert_allclose(got["recurrent"][b, h], want, rtol=1e-11, atol=1e-11)
    if rows is not None:
        want_rows = np.stack([got["quadratic"].reshape(B * H, N, dv)[bh, i] for bh, i in rows])
        np.testing.assert_allclose(got["quadratic_rows"], want_rows, rtol=1e-13, atol=1e-13)
    # one decode step = the first token of the recurrence
    np.testing.assert_allclose(got["decode_out"], got["recurrent"][:, :, 0], rtol=1e-13, atol=1e-13)


def test_sanitizers_do_catch_a_planted_overrun(tmp_path):
    """The check itself is checked: a copy of the oracle whose quadratic form runs one key past the
    causal limit (reading beyond k and v on the last row) must be reported by the sanitized build."""
    src = open(os.path.join(ROOT, "oracle", "leet_oracle.c")).read()
    planted = src.replace("for (long j = 0; j <= i; ++j) {", "for (long j = 0; j <= i + 1; ++j) {")
    assert planted != src
    bad_c = tmp_path / "leet_oracle_planted.c"
    bad_c.write_text(planted)
    exe = str(tmp_path / "oracle_planted")
    res = subprocess.run(["gcc", "-std=c99", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined",
                          "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan", "-o", exe,
                          os.path.join(ROOT, "oracle", "sanitize_driver.c"), str(bad_c), "-lm"],
                         capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    rng = np.random.default_rng(1)
    case = tmp_path / "case.bin"
    with open(case, "wb") as f:
        np.array([1, 1, 5, 4, 4, 0, 0], dtype=np.int64).tofile(f)
        for n in (20, 20, 20, 1):
            rng.standard_normal(n).tofile(f)
    run = subprocess.run([exe, str(case), str(tmp_path / "r.bin")], capture_output=True, text=True,
                         env=dict(os.environ, OMP_NUM_THREADS="1"), timeout=120)
    assert run.returncode != 0 and "AddressSanitizer" in run.stderr
