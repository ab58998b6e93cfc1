"""GPU test of the entry point that allocates nothing (segment states in the library's static
scratch): through the C ABI, against leet_attn_forward_ex on the same inputs -- the same kernels and
the same plan, so bit for bit -- and against the fp64 oracle, on two calls in a row, the second
smaller than the first (the scratch keeps the first call's contents)."""
import ctypes
import sys

import numpy as np
import pytest
import torch

import oracle
from helpers import elementwise_ok, max_rel_err
from paper_2501_02573_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _call_static(B, dq, dk, dv, dg, out, s_in, s_out, segments, dtype_code):
    """Straight through ctypes: raw device pointers, sizes and the current stream."""
    Bn, H, N, d = dq.shape
    vp = ctypes.c_void_p
    st = B.lib.leet_attn_forward_static(vp(dq.data_ptr()), vp(dk.data_ptr()), vp(dv.data_ptr()), vp(dg.data_ptr()),
                                        vp(out.data_ptr()), vp(s_in.data_ptr()) if s_in is not None else None,
                                        vp(s_out.data_ptr()) if s_out is not None else None, segments,
                                        Bn, H, N, d, dtype_code, vp(torch.cuda.current_stream().cuda_stream))
    assert st == B.LEET_OK, B.strerror(st)


CALLS = [
    # two calls in a row, the second smaller: (B, H, N, d, dtype, segments)
    [(2, 8, 4000, 128, "bf16", 6), (1, 3, 700, 128, "bf16", 3)],
    [(1, 12, 3072, 128, "bf16", 0), (1, 5, 3000, 64, "bf16", 0)],      # the library's own plans
    [(2, 4, 1500, 64, "f32", 5), (1, 2, 333, 64, "f32", 2)],
]


@pytest.mark.parametrize("calls", CALLS, ids=lambda c: "then".join("B%d_H%d_N%d_d%d_%s_seg%d" % s for s in c))
def test_forward_static_matches_forward_ex_on_two_calls_in_a_row(calls):
    from paper_2501_02573_amd import binding as B
    assert torch.cuda.is_available()
    for n, (Bn, H, N, d, dtype, segs) in enumerate(calls):
        say(f"case static scratch call {n}: {(Bn, H, N, d, dtype, segs)}")
        code = B.LEET_F32 if dtype == "f32" else B.LEET_BF16
        nseg, _ = B.query_plan(Bn, H, N, d, code, segs)
        assert nseg > 1, "the case must use the scratch"
        assert B.workspace_bytes(Bn, H, N, d, code, segs) <= B.static_scratch_bytes()
        q, k, v, gamma = W.make_custom_forward_inputs(Bn, H, N, d, dtype, seed=5100 + N, gamma=W.make_gamma("pow2:3:9", H))
        rng = np.random.default_rng(N)
        s_in = torch.from_numpy((rng.standard_normal((Bn, H, d, d)) * 0.02).astype(np.float32))
        dq, dk, dv, dg, ds_in = (t.cuda() for t in (q, k, v, gamma, s_in))
        # everything the calls need exists before the entry point under test runs
        out_s = torch.zeros((Bn, H, N, d), dtype=torch.float32, device="cuda")
        S_s = torch.zeros((Bn, H, d, d), dtype=torch.float32, device="cuda")
        ws = torch.empty(B.workspace_bytes(Bn, H, N, d, code, segs), dtype=torch.uint8, device="cuda")
        S_e = torch.zeros_like(S_s)
        torch.cuda.synchronize()
        _call_static(B, dq, dk, dv, dg, out_s, ds_in, S_s, segs, code)
        torch.cuda.synchronize()
        out_e = B.leet_attn_forward_ex(dq, dk, dv, dg, state_in=ds_in, state_out=S_e, workspace=ws, segments=segs)
        torch.cuda.synchronize()
        assert torch.equal(out_s, out_e), "static-scratch output differs from leet_attn_forward_ex"
        assert torch.equal(S_s, S_e), "static-scratch final state differs from leet_attn_forward_ex"
        ref, s_ref = oracle.recurrent(*(W.to_f64(t) for t in (q, k, v, gamma)), state_in=W.to_f64(s_in))
        for got, want, what in ((out_s, ref, "out"), (S_s, s_ref, "final state")):
            err = max_rel_err(got.cpu().numpy(), want)
            say(f"  {what} vs oracle: {err:.3e}")
            assert err <= TOL[dtype] and elementwise_ok(got.cpu().numpy(), want, TOL[dtype])


def test_forward_static_refuses_what_its_scratch_cannot_hold():
    from paper_2501_02573_amd import binding as B
    Bn, H, N, d = 4, 16, 8192, 128
    assert B.workspace_bytes(Bn, H, N, d, B.LEET_BF16, 16) > B.static_scratch_bytes()
    q = torch.zeros((Bn, H, N, d), dtype=torch.bfloat16, device="cuda")
    g = torch.ones(H, device="cuda")
    out = torch.full((Bn, H, N, d), 7.0, device="cuda")
    with pytest.raises(B.LeetAttnError) as ei:
        B.leet_attn_forward_static(q, q, q, g, out, segments=16)
    assert ei.value.status == B.LEET_ERR_SCRATCH_LIMIT
    torch.cuda.synchronize()
    assert torch.all(out == 7.0)
    B.leet_attn_forward_static(q, q, q, g, out, segments=1)   # one segment: no scratch needed
    torch.cuda.synchronize()
    assert torch.all(out == 0.0)
