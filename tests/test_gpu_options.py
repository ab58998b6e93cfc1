"""GPU parity for the optional forms of the path: fp16 inputs, output in the input type,
the 0/1 causal mask (gamma = 1; Section 2.2) and multi-token decode with state hand-off.

Same metric as the main parity tests: max|gpu-ref| / max|ref| per (batch, head), worst head,
against the fp64 oracle on the same seeded inputs (the 16-bit inputs converted exactly).
Tolerances: bf16 inputs 2e-2 and fp32 inputs 1e-4 as everywhere; fp16 inputs 2.5e-3, the bf16
bound scaled by the three extra mantissa bits (the same intermediates -- scores, state, scaled
V -- are rounded to the input type).  An output stored in a 16-bit type adds at most half an
ulp of that type per element (2^-9 of the element for bf16, 2^-12 for fp16), which the same
bounds absorb.
"""
import ctypes
import sys

import numpy as np
import pytest
import torch

import oracle
from helpers import elementwise_ok, max_rel_err
from paper_2501_02573_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2, "f16": 2.5e-3}


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


def check(got, ref, tol, what):
    got = np.asarray(got, dtype=np.float64)
    err = max_rel_err(got, ref)
    say(f"  {what}: max rel err {err:.3e} (tol {tol:.1e})")
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    assert err <= tol, f"{what}: {err} > {tol}"
    assert elementwise_ok(got, ref, tol), f"{what}: element-wise bound violated"


def to_np(t):
    return t.detach().to(torch.float64).cpu().numpy()


OPTION_SHAPES = [
    # B, H, N, d, in dtype, 16-bit output, segments
    (1, 2, 1, 64, "f16", False, 0),
    (2, 3, 200, 128, "f16", False, 0),
    (1, 4, 777, 64, "f16", True, 3),
    (2, 2, 1025, 128, "f16", True, 4),
    (1, 3, 333, 64, "bf16", True, 0),
    (2, 4, 1536, 128, "bf16", True, 3),
    (1, 2, 4096, 128, "f16", False, 0),
]


@pytest.mark.parametrize("kernel", ["auto", "wide", "column-split"])
@pytest.mark.parametrize("shape", OPTION_SHAPES, ids=lambda s: "B%d_H%d_N%d_d%d_%s_out16%d_seg%d" % s)
def test_fp16_inputs_and_16bit_outputs(B, shape, kernel):
    """fp16 and bf16 inputs, fp32 output or output in the input type, through the planner's choice
    and through each kernel family forced."""
    Bn, H, N, d, dtype, out16, segs = shape
    say(f"case shape={shape} kernel={kernel}")
    gamma = torch.tensor(([0.0, 1.0, 0.5, 0.999, 0.9] * 2)[:H], dtype=torch.float32)
    q, k, v, gamma = W.make_custom_forward_inputs(Bn, H, N, d, dtype, seed=2000 + N + d, gamma=gamma)
    rng = np.random.default_rng(N)
    s_in = torch.from_numpy((rng.standard_normal((Bn, H, d, d)) * 0.1).astype(np.float32))
    dq, dk, dv, dg, ds_in = dev(q, k, v, gamma, s_in)
    s_out = torch.empty_like(ds_in)
    q64, k64, v64, g64 = (W.to_f64(t) for t in (q, k, v, gamma))
    odt = W.torch_dtype(dtype) if out16 else torch.float32
    B.set_bf16_kernel({"auto": B.KERNEL_AUTO, "wide": B.KERNEL_WIDE, "column-split": B.KERNEL_COLUMN_SPLIT}[kernel])
    try:
        out = B.leet_attn_forward_v2(dq, dk, dv, dg, state_out=s_out, segments=segs, out_dtype=odt)
        assert out.dtype == odt
        ref, s_ref = oracle.recurrent(q64, k64, v64, g64)
        check(to_np(out), ref, TOL[dtype], "zero state: out")
        check(to_np(s_out), s_ref, TOL[dtype], "zero state: final state")

        out2 = B.leet_attn_forward_v2(dq, dk, dv, dg, state_in=ds_in, state_out=s_out, segments=segs, out_dtype=odt)
        ref2, s_ref2 = oracle.recurrent(q64, k64, v64, g64, state_in=W.to_f64(s_in))
        check(to_np(out2), ref2, TOL[dtype], "with state_in: out")
        check(to_np(s_out), s_ref2, TOL[dtype], "with state_in: final state")

        if out16 and kernel != "auto":
            # the 16-bit output is the fp32 output of the same kernel and plan, rounded to nearest even
            fixed = segs or 2
            o16 = B.leet_attn_forward_v2(dq, dk, dv, dg, state_in=ds_in, segments=fixed, out_dtype=odt)
            o32 = B.leet_attn_forward_v2(dq, dk, dv, dg, state_in=ds_in, segments=fixed)
            assert torch.equal(o32.to(odt), o16), "16-bit output is not the rounded fp32 output"
    finally:
        B.set_bf16_kernel(B.KERNEL_AUTO)


CAUSAL_SHAPES = [
    (1, 2, 130, 64, "f32", 0),
    (2, 2, 1000, 128, "f32", 3),
    (1, 3, 777, 64, "bf16", 2),
    (2, 4, 2048, 128, "bf16", 0),
    (1, 2, 600, 128, "f16", 0),
]


@pytest.mark.parametrize("shape", CAUSAL_SHAPES, ids=lambda s: "B%d_H%d_N%d_d%d_%s_seg%d" % s)
def test_causal_mask_is_gamma_one(B, shape):
    """The 0/1 mask: oracle run with gamma = 1; the GPU gets no gamma at all."""
    Bn, H, N, d, dtype, segs = shape
    say(f"case shape={shape}")
    q, k, v, _ = W.make_custom_forward_inputs(Bn, H, N, d, dtype, seed=3000 + N + d)
    ones = torch.ones(H, dtype=torch.float32)
    dq, dk, dv = dev(q, k, v)
    s_out = torch.empty(Bn, H, d, d, dtype=torch.float32, device="cuda")
    out = B.leet_attn_forward_v2(dq, dk, dv, None, state_out=s_out, segments=segs, mask=B.LEET_MASK_CAUSAL)
    q64, k64, v64, g64 = (W.to_f64(t) for t in (q, k, v, ones))
    ref, s_ref = oracle.recurrent(q64, k64, v64, g64)
    check(to_np(out), ref, TOL[dtype], "causal mask: out")
    check(to_np(s_out), s_ref, TOL[dtype], "causal mask: final state")
    # a gamma that is passed is ignored
    junk = torch.full((H,), 0.25, dtype=torch.float32, device="cuda")
    out_b = B.leet_attn_forward_v2(dq, dk, dv, junk, segments=segs, mask=B.LEET_MASK_CAUSAL)
    assert torch.equal(out, out_b)
    # and the general kernels given gamma = 1 agree to the same tolerance
    out_c = B.leet_attn_forward_v2(dq, dk, dv, ones.cuda(), segments=segs)
    assert max_rel_err(to_np(out_c), to_np(out)) <= TOL[dtype]


@pytest.mark.parametrize("shape", [(1, 3, 777, 64, 2), (2, 4, 2048, 128, 0), (1, 1, 4000, 128, 0), (1, 2, 333, 128, 1)],
                         ids=lambda s: "B%d_H%d_N%d_d%d_seg%d" % s)
def test_causal_mask_on_the_column_split_kernel(B, shape):
    """The 0/1 mask through the column-split bf16 kernel (forced), with an entering state."""
    Bn, H, N, d, segs = shape
    say(f"case shape={shape}")
    q, k, v, _ = W.make_custom_forward_inputs(Bn, H, N, d, "bf16", seed=3100 + N + d)
    ones = torch.ones(H, dtype=torch.float32)
    rng = np.random.default_rng(N)
    s_in = torch.from_numpy((rng.standard_normal((Bn, H, d, d)) * 0.1).astype(np.float32))
    dq, dk, dv, ds_in = dev(q, k, v, s_in)
    s_out = torch.empty_like(ds_in)
    B.set_bf16_kernel(B.KERNEL_COLUMN_SPLIT)
    try:
        assert B.query_plan(Bn, H, N, d, B.LEET_BF16, segs)[1] == B.KERNEL_COLUMN_SPLIT
        out = B.leet_attn_forward_v2(dq, dk, dv, None, state_in=ds_in, state_out=s_out, segments=segs, mask=B.LEET_MASK_CAUSAL)
    finally:
        B.set_bf16_kernel(B.KERNEL_AUTO)
    ref, s_ref = oracle.recurrent(*(W.to_f64(t) for t in (q, k, v, ones)), state_in=W.to_f64(s_in))
    check(to_np(out), ref, TOL["bf16"], "causal mask, column split: out")
    check(to_np(s_out), s_ref, TOL["bf16"], "causal mask, column split: final state")


@pytest.mark.parametrize("dtype,d", [("f16", 128), ("f16", 64), ("bf16", 128)])
def test_decode_v2_dtypes_and_causal_mask(B, dtype, d):
    say(f"case decode_v2 dtype={dtype} d={d}")
    cfg = W.DecodeConfig("t", 3, 5, d, 6, 21, "pow2:1:9", dtype=dtype)
    for mask in (B.LEET_MASK_DECAY, B.LEET_MASK_CAUSAL):
        state0, gamma, steps = W.decode_stream(cfg)
        g_ref = gamma if mask == B.LEET_MASK_DECAY else torch.ones_like(gamma)
        S_ref = W.to_f64(state0); S_gpu = state0.cuda()
        dg = gamma.cuda() if mask == B.LEET_MASK_DECAY else None
        for q, k, v in steps:
            o = B.leet_attn_decode_step_v2(*dev(q, k, v), dg, S_gpu, mask=mask).cpu().numpy()
            o_ref = oracle.decode_step(W.to_f64(q), W.to_f64(k), W.to_f64(v), W.to_f64(g_ref), S_ref)
            assert max_rel_err(o, o_ref) < 1e-5   # fp32 state arithmetic on exactly converted inputs
        assert max_rel_err(S_gpu.cpu().numpy(), S_ref) < 1e-5


@pytest.mark.parametrize("T", [2, 5, 16])
@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64), ("f16", 128)])
def test_multi_token_decode_reuses_the_chunk_kernel(B, dtype, d, T):
    """T tokens at once with the state entering and leaving the call equal T single-token steps."""
    Bn, H, n0 = 4, 3, 100
    say(f"case multi-token decode dtype={dtype} d={d} T={T}")
    q, k, v, gamma = W.make_custom_forward_inputs(Bn, H, n0 + T, d, dtype, seed=500 + T + d)
    dq, dk, dv, dg = dev(q, k, v, gamma)
    S = torch.empty(Bn, H, d, d, dtype=torch.float32, device="cuda")
    head = [t[:, :, :n0].contiguous() for t in (dq, dk, dv)]
    tail = [t[:, :, n0:].contiguous() for t in (dq, dk, dv)]
    B.leet_attn_forward_v2(*head, dg, state_out=S)
    S_steps = S.clone()
    out_T = B.leet_attn_forward_v2(*tail, dg, state_in=S, state_out=S)     # in place
    outs = [B.leet_attn_decode_step_v2(*(t[:, :, i].contiguous() for t in tail), dg, S_steps) for i in range(T)]
    out_steps = torch.stack(outs, dim=2)
    ref, s_ref = oracle.recurrent(*(W.to_f64(t) for t in (q, k, v, gamma)))
    check(to_np(out_T), ref[:, :, n0:], TOL[dtype], "T tokens at once vs oracle")
    check(to_np(out_steps), ref[:, :, n0:], TOL[dtype], "T single steps vs oracle")
    check(to_np(S), s_ref, TOL[dtype], "state after T tokens at once")
    check(to_np(S_steps), s_ref, TOL[dtype], "state after T single steps")


def test_unsupported_combinations_are_rejected_and_write_nothing(B):
    q, k, v, gamma = W.make_custom_forward_inputs(1, 1, 64, 64, "f32", 1)
    dq, dk, dv, dg = dev(q, k, v, gamma)
    vp = ctypes.c_void_p
    out = torch.full((1, 1, 64, 64), 7.0, device="cuda")

    def v2(in_dt, out_dt, mask, g=dg):
        return B.lib.leet_attn_forward_v2(vp(dq.data_ptr()), vp(dk.data_ptr()), vp(dv.data_ptr()),
                                          vp(g.data_ptr()) if g is not None else None, vp(out.data_ptr()),
                                          None, None, None, 0, 0, 1, 1, 64, 64, in_dt, out_dt, mask, None)

    assert v2(B.LEET_F32, B.LEET_BF16, B.LEET_MASK_DECAY) == B.LEET_ERR_UNSUPPORTED    # fp32 in, 16-bit out
    assert v2(B.LEET_BF16, B.LEET_F16, B.LEET_MASK_DECAY) == B.LEET_ERR_UNSUPPORTED    # mixed 16-bit types
    assert v2(B.LEET_F32, B.LEET_F32, 2) == B.LEET_ERR_INVALID_ARG                     # unknown mask
    assert v2(B.LEET_F32, B.LEET_F32, B.LEET_MASK_DECAY, g=None) == B.LEET_ERR_INVALID_ARG  # decay needs gamma
    assert v2(3, B.LEET_F32, B.LEET_MASK_DECAY) == B.LEET_ERR_UNSUPPORTED              # unknown dtype
    # the older entry points do not take fp16
    st = B.lib.leet_attn_forward(vp(dq.data_ptr()), vp(dk.data_ptr()), vp(dv.data_ptr()), vp(dg.data_ptr()),
                                 vp(out.data_ptr()), 1, 1, 64, 64, B.LEET_F16, None)
    assert st == B.LEET_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert torch.all(out == 7.0)


# ---------------------------------------------------------------- row-based prefill (Alg. 1 on the GPU)
RECURRENT_SHAPES = [
    # B, H, N, d, dtype
    (1, 1, 1, 64, "f32"),
    (2, 3, 31, 64, "bf16"),
    (1, 2, 32, 128, "f32"),
    (2, 2, 33, 128, "f16"),
    (1, 5, 777, 128, "bf16"),
    (2, 4, 1000, 64, "f32"),
]


@pytest.mark.parametrize("shape", RECURRENT_SHAPES, ids=lambda s: "B%d_H%d_N%d_d%d_%s" % s)
def test_row_based_prefill_kernel(B, shape):
    """fp32 recurrence on exactly converted inputs: far inside every input-type bound."""
    Bn, H, N, d, dtype = shape
    say(f"case recurrent shape={shape}")
    gamma = torch.tensor(([0.0, 1.0, 0.5, 0.999, 0.9] * 2)[:H], dtype=torch.float32)
    q, k, v, gamma = W.make_custom_forward_inputs(Bn, H, N, d, dtype, seed=4000 + N + d, gamma=gamma)
    rng = np.random.default_rng(N)
    s_in = torch.from_numpy((rng.standard_normal((Bn, H, d, d)) * 0.1).astype(np.float32))
    dq, dk, dv, dg, ds = dev(q, k, v, gamma, s_in)
    q64, k64, v64, g64 = (W.to_f64(t) for t in (q, k, v, gamma))
    s_out = torch.empty_like(ds)
    out = B.leet_attn_forward_recurrent(dq, dk, dv, dg, state_out=s_out)
    ref, s_ref = oracle.recurrent(q64, k64, v64, g64)
    check(to_np(out), ref, 1e-5, "zero state: out")
    check(to_np(s_out), s_ref, 1e-5, "zero state: final state")
    out2 = B.leet_attn_forward_recurrent(dq, dk, dv, dg, state_in=ds, state_out=ds)   # in place
    ref2, s_ref2 = oracle.recurrent(q64, k64, v64, g64, state_in=W.to_f64(s_in))
    check(to_np(out2), ref2, 1e-5, "with state_in: out")
    check(to_np(ds), s_ref2, 1e-5, "with state_in: final state (in place)")
    out3 = B.leet_attn_forward_recurrent(dq, dk, dv, None, mask=B.LEET_MASK_CAUSAL)
    ref3, _ = oracle.recurrent(q64, k64, v64, np.ones(H))
    check(to_np(out3), ref3, 1e-5, "causal mask: out")
    # the chunked path agrees with it to the chunked path's own tolerance
    out4 = B.leet_attn_forward_v2(dq, dk, dv, dg)
    assert max_rel_err(to_np(out4), to_np(out)) <= TOL[dtype]


# ---------------------------------------------------------------- FleetAttention (Eq. "p", Alg. 5 on the GPU)
FLEET_SHAPES = [
    # B, H, N, r, dv, dtype
    (1, 1, 1, 64, 64, "f32"),
    (2, 3, 31, 64, 64, "bf16"),
    (1, 2, 32, 128, 128, "f32"),
    (2, 2, 33, 128, 128, "f16"),
    (1, 5, 777, 128, 128, "bf16"),
    (2, 4, 1000, 64, 64, "f32"),
    (1, 3, 100, 128, 256, "bf16"),
    (2, 2, 65, 128, 256, "f16"),
]


@pytest.mark.parametrize("shape", FLEET_SHAPES, ids=lambda s: "B%d_H%d_N%d_r%d_dv%d_%s" % s)
def test_fleet_attention_kernel(B, shape):
    """fp32 element-wise arithmetic on exactly converted inputs: far inside every input-type bound.
    Compared with the oracle's recurrence (outputs and carried vectors = state rows) and, at the
    small sizes, with the oracle's own rank-sum-of-cumsums form."""
    Bn, H, N, r, dv, dtype = shape
    say(f"case fleet shape={shape}")
    gamma = torch.tensor(([0.0, 1.0, 0.5, 0.999, 0.9] * 2)[:H], dtype=torch.float32)
    q, k, v, gamma = W.make_rd_forward_inputs(Bn, H, N, r, dv, dtype, seed=5000 + N + r, gamma=gamma)
    rng = np.random.default_rng(N)
    s_in = torch.from_numpy((rng.standard_normal((Bn, H, r, dv)) * 0.1).astype(np.float32))
    dq, dk, dv_, dg, ds = dev(q, k, v, gamma, s_in)
    q64, k64, v64, g64 = (W.to_f64(t) for t in (q, k, v, gamma))
    s_out = torch.empty_like(ds)
    out = B.leet_attn_forward_fleet(dq, dk, dv_, dg, state_out=s_out)
    ref, s_ref = oracle.recurrent(q64, k64, v64, g64)
    check(to_np(out), ref, 1e-5, "zero carry: out")
    check(to_np(s_out), s_ref, 1e-5, "zero carry: carried vectors after the last block")
    if N <= 100:
        check(to_np(out), oracle.fleet(q64, k64, v64, g64), 1e-5, "zero carry: out vs the oracle's rank-sum form")
    out2 = B.leet_attn_forward_fleet(dq, dk, dv_, dg, state_in=ds, state_out=ds)   # in place
    ref2, s_ref2 = oracle.recurrent(q64, k64, v64, g64, state_in=W.to_f64(s_in))
    check(to_np(out2), ref2, 1e-5, "with carry in: out")
    check(to_np(ds), s_ref2, 1e-5, "with carry in: carried vectors (in place)")
    out3 = B.leet_attn_forward_fleet(dq, dk, dv_, None, mask=B.LEET_MASK_CAUSAL)
    ref3, _ = oracle.recurrent(q64, k64, v64, np.ones(H))
    check(to_np(out3), ref3, 1e-5, "0/1 mask (plain cumsum): out")
    # the chunked path agrees with it to the chunked path's own tolerance
    out4 = B.leet_attn_forward_rd(dq, dk, dv_, dg)
    assert max_rel_err(to_np(out4), to_np(out)) <= TOL[dtype]


# ---------------------------------------------------------------- rank 128, value width 256 (the paper's usage example)
RD_SHAPES = [
    # B, H, N, dtype, 16-bit output, segments
    (1, 2, 1, "bf16", False, 0),
    (2, 3, 200, "bf16", False, 0),
    (1, 4, 777, "f16", False, 3),
    (2, 2, 1025, "bf16", True, 4),
    (1, 3, 2048, "f16", True, 0),
]


@pytest.fixture(params=["auto", "wide", "column-split"])
def kernel_choice(request, B):
    B.set_bf16_kernel({"auto": B.KERNEL_AUTO, "wide": B.KERNEL_WIDE, "column-split": B.KERNEL_COLUMN_SPLIT}[request.param])
    yield request.param
    B.set_bf16_kernel(B.KERNEL_AUTO)


@pytest.mark.parametrize("shape", RD_SHAPES, ids=lambda s: "B%d_H%d_N%d_%s_out16%d_seg%d" % s)
def test_rank_128_value_width_256(B, shape, kernel_choice):
    Bn, H, N, dtype, out16, segs = shape
    r, dv = 128, 256
    say(f"case r={r} dv={dv} shape={shape} kernel={kernel_choice}")
    gamma = torch.tensor(([0.0, 1.0, 0.5, 0.999, 0.9] * 2)[:H], dtype=torch.float32)
    q, k, v, gamma = W.make_rd_forward_inputs(Bn, H, N + 1, r, dv, dtype, seed=5000 + N, gamma=gamma)
    rng = np.random.default_rng(N)
    s_in = torch.from_numpy((rng.standard_normal((Bn, H, r, dv)) * 0.05).astype(np.float32))
    dq, dk, dv_, dg, ds_in = dev(q, k, v, gamma, s_in)
    head = [t[:, :, :N].contiguous() for t in (dq, dk, dv_)]
    odt = W.torch_dtype(dtype) if out16 else torch.float32
    S = torch.empty_like(ds_in)
    ws = torch.empty(max(B.workspace_bytes_rd(Bn, H, N, r, dv, B.LEET_BF16 if dtype == "bf16" else B.LEET_F16, segs), 1),
                     dtype=torch.uint8, device="cuda")
    out = B.leet_attn_forward_rd(*head, dg, state_in=ds_in, state_out=S, workspace=ws, segments=segs, out_dtype=odt)
    o_last = B.leet_attn_decode_step_rd(dq[:, :, N].contiguous(), dk[:, :, N].contiguous(), dv_[:, :, N].contiguous(), dg, S)
    ref, s_ref = oracle.recurrent(*(W.to_f64(t) for t in (q, k, v, gamma)), state_in=W.to_f64(s_in))
    assert out.shape == (Bn, H, N, dv) and out.dtype == odt
    check(to_np(out), ref[:, :, :N], TOL[dtype], "chunked: out")
    check(to_np(o_last)[:, :, None, :], ref[:, :, N:], TOL[dtype], "decode step after it")
    check(to_np(S), s_ref, TOL[dtype], "state after prefill + one step")
    # the row-based kernel on the same inputs: fp32 recurrence, far tighter
    S2 = torch.empty_like(ds_in)
    out_r = B.leet_attn_forward_recurrent_rd(dq, dk, dv_, dg, state_in=ds_in, state_out=S2)
    check(to_np(out_r), ref, 1e-5, "row-based: out")
    check(to_np(S2), s_ref, 1e-5, "row-based: final state")
    # 0/1 mask
    out_c = B.leet_attn_forward_rd(*head, None, segments=segs, mask=B.LEET_MASK_CAUSAL)
    ref_c, _ = oracle.recurrent(*(W.to_f64(t)[:, :, :N] for t in (q, k, v)), np.ones(H))
    check(to_np(out_c), ref_c, TOL[dtype], "causal mask: out")


def test_rank_value_width_combinations_rejected(B):
    q = torch.zeros(1, 1, 64, 128, device="cuda", dtype=torch.float32)
    v = torch.zeros(1, 1, 64, 256, device="cuda", dtype=torch.float32)
    g = torch.ones(1, device="cuda")
    with pytest.raises(B.LeetAttnError) as ei:        # fp32 inputs: square shapes only
        B.leet_attn_forward_rd(q, q, v, g)
    assert ei.value.status == B.LEET_ERR_UNSUPPORTED
    qb = torch.zeros(1, 1, 64, 64, device="cuda", dtype=torch.bfloat16)
    vb = torch.zeros(1, 1, 64, 128, device="cuda", dtype=torch.bfloat16)
    with pytest.raises(B.LeetAttnError) as ei:        # rank 64 with width 128 is not built
        B.leet_attn_forward_rd(qb, qb, vb, g)
    assert ei.value.status == B.LEET_ERR_UNSUPPORTED
    # 8 segments: 7 boundary states per sequence, kept on half-segments (14 slots) of r x dv floats,
    # and one slot for the copy of the entering state
    assert B.workspace_bytes_rd(1, 32, 32768, 128, 256, B.LEET_BF16, 8) == 32 * 15 * 128 * 256 * 4
    assert B.workspace_bytes_rd(1, 32, 32768, 64, 128, B.LEET_BF16, 8) == 0


def test_decode_store_policies_give_identical_results(B):
    """Cached and streamed state stores differ in memory traffic only."""
    cfg = W.DecodeConfig("t", 4, 6, 128, 5, 33, "pow2:1:9")
    results = []
    try:
        for mode in (B.DECODE_STORE_CACHED, B.DECODE_STORE_STREAM):
            B.set_decode_store(mode)
            state0, gamma, steps = W.decode_stream(cfg)
            S = state0.cuda(); dg = gamma.cuda()
            outs = [B.leet_attn_decode_step(*dev(q, k, v), dg, S).clone() for q, k, v in steps]
            results.append((torch.stack(outs), S.clone()))
    finally:
        B.set_decode_store(B.DECODE_STORE_AUTO)
    assert torch.equal(results[0][0], results[1][0]) and torch.equal(results[0][1], results[1][1])
    state0, gamma, steps = W.decode_stream(cfg)
    S_ref = W.to_f64(state0)
    for n, (q, k, v) in enumerate(steps):
        o_ref = oracle.decode_step(W.to_f64(q), W.to_f64(k), W.to_f64(v), W.to_f64(gamma), S_ref)
        assert max_rel_err(to_np(results[1][0][n]), o_ref) < 1e-5
    assert max_rel_err(to_np(results[1][1]), S_ref) < 1e-5


def test_usage_example_shape_heads32_rank128_dim256(B):
    """The shape of the paper's usage example (Section 4): heads 32, rank 128, dim 256; N = 8192, batch 1,
    in the launch configuration the library picks by itself."""
    Bn, H, N, r, dv = 1, 32, 8192, 128, 256
    say(f"case usage-example shape B={Bn} H={H} N={N} r={r} dv={dv}")
    q, k, v, gamma = W.make_rd_forward_inputs(Bn, H, N, r, dv, "bf16", seed=77, gamma=W.make_gamma("pow2:5:10", H))
    out = B.leet_attn_forward_rd(*dev(q, k, v, gamma))
    torch.cuda.synchronize()
    ref, _ = oracle.recurrent(*(W.to_f64(t) for t in (q, k, v, gamma)))
    check(to_np(out), ref, TOL["bf16"], "out (all elements)")


# ---------------------------------------------------------------- seeded random legal shapes and options
def _random_cases(n, seed=2024):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        dtype = ["bf16", "f16", "f32"][int(rng.integers(0, 3))]
        d = int(rng.choice([64, 128]))
        dv = 256 if (d == 128 and dtype != "f32" and rng.random() < 0.25) else d
        Bn, H = int(rng.integers(1, 4)), int(rng.integers(1, 6))
        N = int(rng.choice([1, 17, 64, 65, 127, 128, 300, 511, 900, 1500]))
        segs = int(rng.choice([0, 0, 1, 2, 3, 7]))
        out16 = bool(dtype != "f32" and rng.random() < 0.4)
        causal = bool(rng.random() < 0.25)
        with_state = bool(rng.random() < 0.5)
        cases.append((i, Bn, H, N, d, dv, dtype, segs, out16, causal, with_state))
    return cases


@pytest.mark.parametrize("case", _random_cases(24), ids=lambda c: "n%d_B%d_H%d_N%d_r%d_dv%d_%s_seg%d_o%d_c%d_s%d" % c)
def test_random_legal_shapes_and_options(B, case):
    i, Bn, H, N, d, dv, dtype, segs, out16, causal, with_state = case
    say(f"case random {case}")
    rng = np.random.default_rng(100 + i)
    gamma = torch.from_numpy(rng.uniform(0.0, 1.0, size=H).astype(np.float32))
    q, k, v, gamma = W.make_rd_forward_inputs(Bn, H, N, d, dv, dtype, seed=7000 + i, gamma=gamma)
    s_in = torch.from_numpy((rng.standard_normal((Bn, H, d, dv)) * 0.03).astype(np.float32)) if with_state else None
    dq, dk, dvv = dev(q, k, v)
    dg = None if causal else gamma.cuda()
    ds_in = s_in.cuda() if with_state else None
    S = torch.empty(Bn, H, d, dv, dtype=torch.float32, device="cuda")
    odt = W.torch_dtype(dtype) if out16 else torch.float32
    out = B.leet_attn_forward_rd(dq, dk, dvv, dg, state_in=ds_in, state_out=S, segments=segs, out_dtype=odt,
                                 mask=B.LEET_MASK_CAUSAL if causal else B.LEET_MASK_DECAY)
    g_ref = np.ones(H) if causal else W.to_f64(gamma)
    ref, s_ref = oracle.recurrent(W.to_f64(q), W.to_f64(k), W.to_f64(v), g_ref,
                                  state_in=None if s_in is None else W.to_f64(s_in))
    check(to_np(out), ref, TOL[dtype], "out")
    check(to_np(S), s_ref, TOL[dtype], "final state")


def _random_planned_cases(n, seed=4242):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        dtype = ["bf16", "f16"][int(rng.integers(0, 2))]
        d = int(rng.choice([64, 128]))
        dv = 256 if (d == 128 and rng.random() < 0.3) else d
        Bn, H = int(rng.integers(1, 3)), int(rng.choice([1, 2, 3, 5, 8, 12, 20]))
        N = int(rng.choice([2000, 3333, 4096, 6000, 9999, 16384]))
        out16 = bool(rng.random() < 0.3)
        cases.append((i, Bn, H, N, d, dv, dtype, out16))
    return cases


@pytest.mark.parametrize("case", _random_planned_cases(12), ids=lambda c: "n%d_B%d_H%d_N%d_r%d_dv%d_%s_o%d" % c)
def test_random_longer_shapes_under_the_planner(B, case):
    """Longer sequences with few to some heads: whatever (kernel, segment count) the planner picks
    (many segments of either kernel), with an entering state and the final state checked."""
    i, Bn, H, N, d, dv, dtype, out16 = case
    code = B.LEET_BF16 if dtype == "bf16" else B.LEET_F16
    say(f"case planned {case} plan (segments, kernel)={B.query_plan_rd(Bn, H, N, d, dv, code)}")
    rng = np.random.default_rng(300 + i)
    gamma = torch.from_numpy((1.0 - 2.0 ** -rng.uniform(2.0, 10.0, size=H)).astype(np.float32))
    q, k, v, gamma = W.make_rd_forward_inputs(Bn, H, N, d, dv, dtype, seed=9000 + i, gamma=gamma)
    s_in = torch.from_numpy((rng.standard_normal((Bn, H, d, dv)) * 0.02).astype(np.float32))
    dq, dk, dvv, dg, ds_in = dev(q, k, v, gamma, s_in)
    S = torch.empty(Bn, H, d, dv, dtype=torch.float32, device="cuda")
    odt = W.torch_dtype(dtype) if out16 else torch.float32
    out = B.leet_attn_forward_rd(dq, dk, dvv, dg, state_in=ds_in, state_out=S, out_dtype=odt)
    ref, s_ref = oracle.recurrent(*(W.to_f64(t) for t in (q, k, v, gamma)), state_in=W.to_f64(s_in))
    check(to_np(out), ref, TOL[dtype], "out")
    check(to_np(S), s_ref, TOL[dtype], "final state")


@pytest.mark.parametrize("out16", [False, True])
def test_caller_workspace_sized_by_the_query_fits_every_output_type(B, out16):
    """The workspace query has no output-type argument: the size it reports must serve a call with
    fp32 output and one with 16-bit output alike (the plan does not depend on the output type)."""
    Bn, H, N, d = 1, 4, 4096, 128
    nseg, _ = B.query_plan(Bn, H, N, d, B.LEET_BF16)
    assert nseg > 1
    need = B.workspace_bytes(Bn, H, N, d, B.LEET_BF16)
    assert need > 0
    q, k, v, gamma = W.make_custom_forward_inputs(Bn, H, N, d, "bf16", seed=61)
    dq, dk, dv, dg = dev(q, k, v, gamma)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    out = B.leet_attn_forward_v2(dq, dk, dv, dg, workspace=ws, out_dtype=torch.bfloat16 if out16 else torch.float32)
    ref, _ = oracle.recurrent(*(W.to_f64(t) for t in (q, k, v, gamma)))
    check(to_np(out), ref, TOL["bf16"], "out with a caller workspace of the queried size")
    with pytest.raises(B.LeetAttnError):   # one byte short is refused before anything is launched
        B.leet_attn_forward_v2(dq, dk, dv, dg, workspace=ws[: need - 256], out_dtype=torch.bfloat16 if out16 else torch.float32)
