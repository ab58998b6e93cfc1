"""GPU parity: the HIP path through the C ABI against the fp64 oracle, same seeded inputs.

Tolerances (primary metric: max|gpu-ref| / max|ref| per (batch, head), worst head):
fp32 inputs 1e-4, bf16 inputs 2e-2 (fp32 accumulate).  The secondary element-wise
check |gpu-ref| <= tol (|ref| + rms(ref)) guards against isolated bad elements.
"""
import sys

import numpy as np
import pytest
import torch

import oracle
from helpers import elementwise_ok, elementwise_ok_windowed, max_rel_err
from paper_2501_02573_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module")
def B():
    from paper_2501_02573_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return binding


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def dev(*ts):
    return tuple(t.cuda() for t in ts)


def check(got, ref, dtype, what):
    err = max_rel_err(got, ref)
    say(f"  {what}: max rel err {err:.3e} (tol {TOL[dtype]:.0e})")
    assert np.isfinite(np.asarray(got)).all(), f"{what}: non-finite output"
    assert err <= TOL[dtype], f"{what}: {err} > {TOL[dtype]}"
    assert elementwise_ok(got, ref, TOL[dtype]), f"{what}: element-wise bound violated"


# ---------------------------------------------------------------- benchmark configurations
def test_config1_tiny_f32_both_forms(B):
    cfg = W.CONFIG1
    say(f"case {cfg}")
    q, k, v, gamma = W.make_forward_inputs(cfg)
    out = B.leet_attn_forward(*dev(q, k, v, gamma)).cpu().numpy()
    q64, k64, v64, g64 = (W.to_f64(t) for t in (q, k, v, gamma))
    check(out, oracle.quadratic(q64, k64, v64, g64), cfg.dtype, "vs quadratic")
    check(out, oracle.recurrent(q64, k64, v64, g64)[0], cfg.dtype, "vs recurrent")


def test_config2_small_f32(B):
    cfg = W.CONFIG2
    say(f"case {cfg}")
    q, k, v, gamma = W.make_forward_inputs(cfg)
    out = B.leet_attn_forward(*dev(q, k, v, gamma)).cpu().numpy()
    q64, k64, v64, g64 = (W.to_f64(t) for t in (q, k, v, gamma))
    check(out, oracle.recurrent(q64, k64, v64, g64)[0], cfg.dtype, "vs recurrent")
    check(out, oracle.quadratic(q64, k64, v64, g64), cfg.dtype, "vs quadratic")


def _sample_rows(cfg, per_head=6, seed=99):
    rng = np.random.default_rng(seed)
    rows = []
    for bh in range(cfg.B * cfg.H):
        picks = {0, cfg.N - 1, 63, 64}
        while len(picks) < per_head + 4:
            picks.add(int(rng.integers(0, cfg.N)))
        rows += [[bh, i] for i in sorted(picks)]
    return np.array(rows)


@pytest.mark.parametrize("cfg", [W.CONFIG3, W.CONFIG4], ids=lambda c: c.name)
def test_full_size_bf16_configs(B, cfg):
    """Full benchmark sizes in the launch configuration bench.py times (library-chosen segments)."""
    say(f"case {cfg}")
    q, k, v, gamma = W.make_forward_inputs(cfg)
    dq, dk, dv, dg = dev(q, k, v, gamma)
    out_d = B.leet_attn_forward(dq, dk, dv, dg)
    torch.cuda.synchronize()
    out = out_d.cpu().numpy()
    del out_d
    q64, k64, v64, g64 = (W.to_f64(t) for t in (q, k, v, gamma))
    ref, _ = oracle.recurrent(q64, k64, v64, g64)
    check(out, ref, cfg.dtype, "vs recurrent (all elements)")
    rows = _sample_rows(cfg)
    quad = oracle.quadratic_rows(q64, k64, v64, g64, rows)
    got = np.stack([out.reshape(cfg.B * cfg.H, cfg.N, cfg.d)[bh, i] for bh, i in rows])
    scale = np.abs(ref).reshape(cfg.B * cfg.H, -1).max(axis=1)[rows[:, 0]][:, None]
    err = float((np.abs(got - quad) / scale).max())
    say(f"  vs quadratic on {len(rows)} sampled rows: {err:.3e}")
    assert err <= TOL[cfg.dtype]


def test_config5_decode_256_steps(B):
    cfg = W.CONFIG5
    say(f"case {cfg}")
    state0, gamma, steps = W.decode_stream(cfg)
    S_ref = W.to_f64(state0)
    g64 = W.to_f64(gamma)
    S_gpu = state0.cuda()
    dg = gamma.cuda()
    worst = 0.0
    for n, (q, k, v) in enumerate(steps):
        o = B.leet_attn_decode_step(*dev(q, k, v), dg, S_gpu).cpu().numpy()
        o_ref = oracle.decode_step(W.to_f64(q), W.to_f64(k), W.to_f64(v), g64, S_ref)
        err = max_rel_err(o, o_ref)
        worst = max(worst, err)
        assert err <= TOL["bf16"], f"step {n}: {err}"
    say(f"  worst step output err {worst:.3e}")
    check(S_gpu.cpu().numpy(), S_ref, "bf16", "final state")
    # fp32 state arithmetic on bf16-exact inputs: far tighter than the bf16 bound
    assert worst < 1e-4 and max_rel_err(S_gpu.cpu().numpy(), S_ref) < 1e-4


# ---------------------------------------------------------------- shapes, tails, segments, degenerate gammas
SHAPES = [
    # B, H, N, d, dtype, segments
    (1, 1, 1, 64, "f32", 0),
    (1, 2, 63, 64, "f32", 0),
    (2, 1, 64, 64, "bf16", 0),
    (1, 2, 65, 128, "f32", 0),
    (1, 3, 200, 128, "bf16", 0),
    (2, 3, 777, 64, "bf16", 3),
    (1, 4, 777, 128, "bf16", 4),
    (1, 4, 1000, 64, "f32", 5),
    (1, 2, 1025, 128, "f32", 2),
    (1, 2, 130, 64, "f32", 50),      # more segments requested than chunks: clamped
    (3, 5, 1536, 128, "bf16", 0),
    (1, 1, 4096, 128, "bf16", 16),
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "B%d_H%d_N%d_d%d_%s_seg%d" % s)
def test_shapes_tails_segments(B, shape):
    Bn, H, N, d, dtype, segs = shape
    say(f"case shape={shape}")
    gamma = torch.tensor(([0.0, 1.0, 0.5, 0.999, 0.9] * 2)[:H], dtype=torch.float32)
    q, k, v, gamma = W.make_custom_forward_inputs(Bn, H, N, d, dtype, seed=1000 + N + d, gamma=gamma)
    rng = np.random.default_rng(N)
    s_in = torch.from_numpy((rng.standard_normal((Bn, H, d, d)) * 0.1).astype(np.float32))
    dq, dk, dv, dg, ds_in = dev(q, k, v, gamma, s_in)
    s_out = torch.empty_like(ds_in)
    q64, k64, v64, g64 = (W.to_f64(t) for t in (q, k, v, gamma))

    out = B.leet_attn_forward_ex(dq, dk, dv, dg, state_out=s_out, segments=segs).cpu().numpy()
    ref, s_ref = oracle.recurrent(q64, k64, v64, g64)
    check(out, ref, dtype, "zero state: out")
    check(s_out.cpu().numpy(), s_ref, dtype, "zero state: final state")

    ws_bytes = B.workspace_bytes(Bn, H, N, d, B.LEET_F32 if dtype == "f32" else B.LEET_BF16, segs)
    ws = torch.empty(max(ws_bytes, 1), dtype=torch.uint8, device="cuda")
    out2 = B.leet_attn_forward_ex(dq, dk, dv, dg, state_in=ds_in, state_out=s_out, workspace=ws,
                                  segments=segs).cpu().numpy()
    ref2, s_ref2 = oracle.recurrent(q64, k64, v64, g64, state_in=W.to_f64(s_in))
    check(out2, ref2, dtype, "with state_in: out")
    check(s_out.cpu().numpy(), s_ref2, dtype, "with state_in: final state")

    if segs == 0:
        out3 = B.leet_attn_forward(dq, dk, dv, dg).cpu().numpy()
        assert np.array_equal(out3, out), "forward and forward_ex(zero state) differ"


def test_segment_count_does_not_change_the_result_beyond_rounding(B):
    q, k, v, gamma = W.make_custom_forward_inputs(1, 4, 2048, 128, "bf16", 5, W.make_gamma("pow2:5:10", 4))
    dq, dk, dv, dg = dev(q, k, v, gamma)
    ref, _ = oracle.recurrent(*(W.to_f64(t) for t in (q, k, v, gamma)))
    for segs in (1, 2, 7, 32):
        say(f"case segments={segs}")
        out = B.leet_attn_forward_ex(dq, dk, dv, dg, segments=segs).cpu().numpy()
        check(out, ref, "bf16", f"segments={segs}")


# ---------------------------------------------------------------- prefill -> decode hand-off
@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64)])
@pytest.mark.parametrize("n0", [128, 129])
def test_prefill_then_decode_matches_one_prefill(B, dtype, d, n0):
    """State carried from chunked prefill into decode steps: prefill(n0) + T steps == prefill(n0 + T)."""
    Bn, H, T = 2, 3, 9
    say(f"case dtype={dtype} d={d} n0={n0}")
    q, k, v, gamma = W.make_custom_forward_inputs(Bn, H, n0 + T, d, dtype, seed=77 + n0)
    dq, dk, dv, dg = dev(q, k, v, gamma)
    S = torch.empty(Bn, H, d, d, dtype=torch.float32, device="cuda")
    B.leet_attn_forward_ex(dq[:, :, :n0].contiguous(), dk[:, :, :n0].contiguous(),
                           dv[:, :, :n0].contiguous(), dg, state_out=S)
    outs = []
    for i in range(n0, n0 + T):
        outs.append(B.leet_attn_decode_step_ex(dq[:, :, i].contiguous(), dk[:, :, i].contiguous(),
                                               dv[:, :, i].contiguous(), dg, S).cpu().numpy())
    dec = np.stack(outs, axis=2)
    S_full = torch.empty_like(S)
    full = B.leet_attn_forward_ex(dq, dk, dv, dg, state_out=S_full).cpu().numpy()
    ref, s_ref = oracle.recurrent(*(W.to_f64(t) for t in (q, k, v, gamma)))
    tail_ref = ref[:, :, n0:]
    check(dec, tail_ref, dtype, "decode outputs vs oracle")
    check(full[:, :, n0:], tail_ref, dtype, "prefill tail vs oracle")
    check(S.cpu().numpy(), s_ref, dtype, "state after decode vs oracle")
    check(S_full.cpu().numpy(), s_ref, dtype, "state after prefill vs oracle")
    # the two GPU routes agree with each other to the same tolerance
    assert max_rel_err(dec, full[:, :, n0:]) <= TOL[dtype]
    assert max_rel_err(S.cpu().numpy(), S_full.cpu().numpy()) <= TOL[dtype]


def test_decode_f32_and_d64(B):
    for d, dtype in ((64, "bf16"), (64, "f32"), (128, "f32")):
        say(f"case decode d={d} dtype={dtype}")
        cfg = W.DecodeConfig("t", 3, 5, d, 7, 11, "pow2:1:9", dtype=dtype)
        state0, gamma, steps = W.decode_stream(cfg)
        S_ref = W.to_f64(state0); S_gpu = state0.cuda(); dg = gamma.cuda()
        for q, k, v in steps:
            o = B.leet_attn_decode_step_ex(*dev(q, k, v), dg, S_gpu).cpu().numpy()
            o_ref = oracle.decode_step(W.to_f64(q), W.to_f64(k), W.to_f64(v), W.to_f64(gamma), S_ref)
            assert max_rel_err(o, o_ref) < 1e-5
        assert max_rel_err(S_gpu.cpu().numpy(), S_ref) < 1e-5


# ---------------------------------------------------------------- determinism and error paths on the device
def test_bitwise_determinism(B):
    q, k, v, gamma = W.make_custom_forward_inputs(2, 4, 1500, 128, "bf16", 3)
    dq, dk, dv, dg = dev(q, k, v, gamma)
    a = B.leet_attn_forward(dq, dk, dv, dg).cpu()
    b = B.leet_attn_forward(dq, dk, dv, dg).cpu()
    assert torch.equal(a, b)


def test_errors_write_nothing(B):
    q, k, v, gamma = W.make_custom_forward_inputs(1, 1, 64, 64, "f32", 1)
    dq, dk, dv, dg = dev(q, k, v, gamma)
    out = torch.full((1, 1, 64, 64), 7.0, device="cuda")
    import ctypes
    st = B.lib.leet_attn_forward(ctypes.c_void_p(dq.data_ptr()), ctypes.c_void_p(dk.data_ptr()),
                                 ctypes.c_void_p(dv.data_ptr()), ctypes.c_void_p(dg.data_ptr()),
                                 ctypes.c_void_p(out.data_ptr()), 1, 1, 64, 96, B.LEET_F32, None)
    assert st == B.LEET_ERR_UNSUPPORTED
    ws = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.LeetAttnError) as ei:   # workspace too small for 2 segments
        q2, k2, v2, g2 = dev(*W.make_custom_forward_inputs(1, 1, 256, 64, "f32", 2))
        B.leet_attn_forward_ex(q2, k2, v2, g2, workspace=ws, segments=2)
    assert ei.value.status == B.LEET_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert torch.all(out == 7.0)


# ---------------------------------------------------------------- the column-split bf16 kernel
@pytest.fixture
def column_split(B):
    B.set_bf16_kernel(B.KERNEL_COLUMN_SPLIT)
    yield B
    B.set_bf16_kernel(B.KERNEL_AUTO)


@pytest.fixture
def wide_only(B):
    B.set_bf16_kernel(B.KERNEL_WIDE)
    yield B
    B.set_bf16_kernel(B.KERNEL_AUTO)


def test_wide_kernel_headline_config(wide_only):
    """The automatic choice runs the column-split kernel on config 3; the wide path must hold there too."""
    B = wide_only
    cfg = W.CONFIG3
    assert B.query_plan(cfg.B, cfg.H, cfg.N, cfg.d, B.LEET_BF16) == (4, B.KERNEL_WIDE)
    say(f"case wide {cfg}")
    q, k, v, gamma = W.make_forward_inputs(cfg)
    out = B.leet_attn_forward(*dev(q, k, v, gamma)).cpu().numpy()
    ref, _ = oracle.recurrent(*(W.to_f64(t) for t in (q, k, v, gamma)))
    check(out, ref, "bf16", "vs recurrent (all elements)")


def test_automatic_kernel_choice_with_state_hand_off(B):
    """A shape for which the planner picks the column-split kernel on whole sequences: ragged length, state in and out,
    continued by a decode step; compared with the oracle and with the wide path."""
    Bn, H, N, d = 4, 16, 1100, 128
    assert B.get_bf16_kernel() == B.KERNEL_AUTO
    assert B.query_plan(Bn, H, N, d, B.LEET_BF16) == (1, B.KERNEL_COLUMN_SPLIT)
    q, k, v, gamma = W.make_custom_forward_inputs(Bn, H, N + 1, d, "bf16", seed=31, gamma=W.make_gamma("pow2:2:9", H))
    rng = np.random.default_rng(5)
    # entering state of the size a steady state has (with a much larger one the fast-decaying heads'
    # first outputs dwarf the rest of the sequence, and the per-head rms of the element-wise check
    # no longer reflects the scale the rounding errors come from)
    s_in = torch.from_numpy((rng.standard_normal((Bn, H, d, d)) * 0.02).astype(np.float32))
    dq, dk, dv, dg, ds_in = dev(q, k, v, gamma, s_in)
    head = [t[:, :, :N].contiguous() for t in (dq, dk, dv)]
    S = torch.empty_like(ds_in)
    out = B.leet_attn_forward_ex(*head, dg, state_in=ds_in, state_out=S).cpu().numpy()
    o_last = B.leet_attn_decode_step(dq[:, :, N].contiguous(), dk[:, :, N].contiguous(), dv[:, :, N].contiguous(), dg, S)
    ref, s_ref = oracle.recurrent(*(W.to_f64(t) for t in (q, k, v, gamma)), state_in=W.to_f64(s_in))
    check(out, ref[:, :, :N], "bf16", "automatic choice: out")
    check(o_last.cpu().numpy()[:, :, None, :], ref[:, :, N:], "bf16", "decode step after it")
    check(S.cpu().numpy(), s_ref, "bf16", "state after prefill + one step")
    B.set_bf16_kernel(B.KERNEL_WIDE)
    try:
        out_w = B.leet_attn_forward_ex(*head, dg, state_in=ds_in).cpu().numpy()
    finally:
        B.set_bf16_kernel(B.KERNEL_AUTO)
    assert max_rel_err(out_w, out) <= TOL["bf16"]


COOP_SHAPES = [
    (1, 1, 1, 128, 0), (2, 1, 64, 64, 0), (1, 3, 200, 128, 0), (2, 3, 777, 64, 3), (1, 4, 777, 128, 4),
    (3, 5, 1536, 128, 0), (1, 9, 1000, 128, 2), (1, 1, 4096, 128, 16),
    # many workgroups: several rounds per compute unit, group counts that are not multiples of 8
    (3, 100, 130, 64, 0), (2, 70, 200, 128, 2), (1, 37, 321, 128, 3),
]


@pytest.mark.parametrize("shape", COOP_SHAPES, ids=lambda s: "B%d_H%d_N%d_d%d_seg%d" % s)
def test_column_split_kernel_shapes(column_split, shape):
    """Same oracle, same tolerances, for the kernel that gives each 32-column slice its own workgroup."""
    B = column_split
    Bn, H, N, d, segs = shape
    say(f"case column-split shape={shape}")
    gamma = torch.tensor(([0.0, 1.0, 0.5, 0.999, 0.9] * (H // 5 + 1))[:H], dtype=torch.float32)
    q, k, v, gamma = W.make_custom_forward_inputs(Bn, H, N, d, "bf16", seed=2000 + N + d, gamma=gamma)
    rng = np.random.default_rng(N + 1)
    # Entering state: its bf16 rounding inside the kernels is the largest error of the first tokens of
    # a fast-decaying head.  At scale 0.1 the element-wise check holds with little room (with millions
    # of outputs a 3.6-sigma element of a gamma = 0.5 head exceeded its bound by 0.5 % -- the wide
    # kernel gives the same value), so the big shapes enter with the size a steady state has.
    scale = 0.1 if Bn * H * N * d < 1_000_000 else 0.02
    s_in = torch.from_numpy((rng.standard_normal((Bn, H, d, d)) * scale).astype(np.float32))
    dq, dk, dv, dg, ds_in = dev(q, k, v, gamma, s_in)
    s_out = torch.empty_like(ds_in)
    q64, k64, v64, g64 = (W.to_f64(t) for t in (q, k, v, gamma))
    out = B.leet_attn_forward_ex(dq, dk, dv, dg, state_in=ds_in, state_out=s_out, segments=segs).cpu().numpy()
    ref, s_ref = oracle.recurrent(q64, k64, v64, g64, state_in=W.to_f64(s_in))
    check(out, ref, "bf16", "out")
    check(s_out.cpu().numpy(), s_ref, "bf16", "final state")


def test_column_split_kernel_headline_config(column_split):
    B = column_split
    cfg = W.CONFIG3
    say(f"case column-split {cfg}")
    q, k, v, gamma = W.make_forward_inputs(cfg)
    out = B.leet_attn_forward(*dev(q, k, v, gamma)).cpu().numpy()
    ref, _ = oracle.recurrent(*(W.to_f64(t) for t in (q, k, v, gamma)))
    check(out, ref, cfg.dtype, "vs recurrent (all elements)")


@pytest.mark.parametrize("kernel", ["auto", "wide", "column-split"])
def test_large_entering_state_at_the_headline_size(B, kernel):
    """Config 3's shape entered with a state of scale 0.1 (the decode benchmark's), five times a steady
    state: the first tokens of the fast-decaying heads are then far larger than the rest of the head.
    Primary metric as everywhere; the element-wise bound is held against the rms of the 64-token
    window the element sits in (the scale its rounding errors come from), for both kernels."""
    cfg = W.CONFIG3
    choice = {"auto": B.KERNEL_AUTO, "wide": B.KERNEL_WIDE, "column-split": B.KERNEL_COLUMN_SPLIT}[kernel]
    say(f"case large entering state {cfg} kernel={kernel}")
    q, k, v, gamma = W.make_forward_inputs(cfg)
    rng = np.random.default_rng(2025)
    s_in = torch.from_numpy((rng.standard_normal((cfg.B, cfg.H, cfg.d, cfg.d)) * 0.1).astype(np.float32))
    dq, dk, dv, dg, ds_in = dev(q, k, v, gamma, s_in)
    S = torch.empty_like(ds_in)
    out = B.leet_attn_forward_v3(dq, dk, dv, dg, state_in=ds_in, state_out=S, kernel=choice).cpu().numpy()
    ref, s_ref = oracle.recurrent(*(W.to_f64(t) for t in (q, k, v, gamma)), state_in=W.to_f64(s_in))
    err = max_rel_err(out, ref)
    say(f"  out: max rel err {err:.3e}")
    assert err <= TOL["bf16"]
    assert elementwise_ok_windowed(out, ref, TOL["bf16"]), "element-wise bound (64-token windows) violated"
    check(S.cpu().numpy(), s_ref, "bf16", "final state")


# ---------------------------------------------------------------- HIP graph capture
def test_prefill_and_decode_replay_from_a_hip_graph(B):
    """The library's launches can be captured; every replay, with eager work in between, equals eager."""
    q, k, v, gamma = W.make_custom_forward_inputs(2, 4, 1100, 128, "bf16", 9)
    dq, dk, dv, dg = dev(q, k, v, gamma)
    S0 = torch.empty(2, 4, 128, 128, dtype=torch.float32, device="cuda")
    eager = B.leet_attn_forward_ex(dq, dk, dv, dg, state_out=S0, segments=3).clone()   # also sizes the workspace
    q1, k1, v1 = (t[:, :, 0].contiguous() for t in (dq, dk, dv))
    S_e = S0.clone()
    o_e = B.leet_attn_decode_step(q1, k1, v1, dg, S_e).clone()
    torch.cuda.synchronize()

    out = torch.zeros_like(eager)
    S = torch.zeros_like(S0)
    o1 = torch.zeros_like(o_e)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        B.leet_attn_forward_ex(dq, dk, dv, dg, out=out, state_out=S, segments=3)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.leet_attn_forward_ex(dq, dk, dv, dg, out=out, state_out=S, segments=3)
        B.leet_attn_decode_step(q1, k1, v1, dg, S, o1)
    for rep in range(3):
        out.zero_(); S.zero_(); o1.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), f"replay {rep}: prefill output differs from eager"
        assert torch.equal(S, S_e), f"replay {rep}: state differs from eager"
        assert torch.equal(o1, o_e), f"replay {rep}: decode output differs from eager"
        # eager work of the program between replays
        other = B.leet_attn_forward_ex(dq, dk, dv, dg, segments=2)   # other segment count: equal up to rounding
        assert max_rel_err(other.cpu().numpy(), eager.cpu().numpy()) < TOL["bf16"]


# ---------------------------------------------------------------- extremes of the launch geometry
def test_one_very_long_sequence(B):
    """One (batch, head) of 262144 tokens: 4096 chunks cut into many segments, a long scan."""
    N, d = 262144, 64
    say(f"case long sequence N={N} d={d}")
    nseg, kern = B.query_plan(1, 1, N, d, B.LEET_BF16)
    assert nseg >= 32
    q, k, v, gamma = W.make_custom_forward_inputs(1, 1, N, d, "bf16", seed=9, gamma=torch.tensor([0.999]))
    S = torch.empty(1, 1, d, d, dtype=torch.float32, device="cuda")
    out = B.leet_attn_forward_ex(*dev(q, k, v, gamma), state_out=S).cpu().numpy()
    ref, s_ref = oracle.recurrent(*(W.to_f64(t) for t in (q, k, v, gamma)))
    check(out, ref, "bf16", "out")
    check(S.cpu().numpy(), s_ref, "bf16", "final state")


PLANNED_SHAPES = [
    (1, 1, 3000, 128), (1, 2, 1000, 128), (1, 3, 8192, 64), (2, 2, 5000, 128), (1, 5, 2100, 64),
    (1, 8, 1536, 128), (1, 12, 3072, 128), (1, 1, 300, 128), (1, 24, 3072, 64),
]


@pytest.mark.parametrize("shape", PLANNED_SHAPES, ids=lambda s: "B%d_H%d_N%d_d%d" % s)
def test_few_sequences_with_the_plans_the_library_picks(B, shape):
    """Few (batch, head) pairs: the planner cuts them into many short segments, mostly of the
    column-split kernel.  State in and out, ragged lengths, the library's own plan."""
    Bn, H, N, d = shape
    plan = B.query_plan(Bn, H, N, d, B.LEET_BF16)
    say(f"case few sequences shape={shape} plan (segments, kernel)={plan}")
    q, k, v, gamma = W.make_custom_forward_inputs(Bn, H, N, d, "bf16", seed=700 + N, gamma=W.make_gamma("pow2:3:10", H) if H > 1 else torch.tensor([0.998]))
    rng = np.random.default_rng(N + 7)
    s_in = torch.from_numpy((rng.standard_normal((Bn, H, d, d)) * 0.02).astype(np.float32))
    dq, dk, dv, dg, ds_in = dev(q, k, v, gamma, s_in)
    S = torch.empty_like(ds_in)
    out = B.leet_attn_forward_ex(dq, dk, dv, dg, state_in=ds_in, state_out=S).cpu().numpy()
    ref, s_ref = oracle.recurrent(*(W.to_f64(t) for t in (q, k, v, gamma)), state_in=W.to_f64(s_in))
    check(out, ref, "bf16", "out")
    check(S.cpu().numpy(), s_ref, "bf16", "final state")


def test_many_short_sequences(B):
    """2560 (batch, head) pairs of 100 tokens: no segments, one ragged pair of chunks per workgroup."""
    Bn, H, N, d = 64, 40, 100, 128
    say(f"case many sequences B={Bn} H={H} N={N}")
    assert B.query_plan(Bn, H, N, d, B.LEET_BF16) == (1, B.KERNEL_WIDE)
    q, k, v, gamma = W.make_custom_forward_inputs(Bn, H, N, d, "bf16", seed=10, gamma=W.make_gamma("pow2:1:10", H))
    out = B.leet_attn_forward(*dev(q, k, v, gamma)).cpu().numpy()
    ref, _ = oracle.recurrent(*(W.to_f64(t) for t in (q, k, v, gamma)))
    check(out, ref, "bf16", "out")
