"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "leet_attn.h")
HEADERS = [HEADER, os.path.join(ROOT, "include", "leet_attn_bench.h")]   # the boundary, and the measurement aids
LIB = os.path.join(ROOT, "paper_2501_02573_amd", "libleet_attn.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2501_02573_amd import build
        build.build()
    from paper_2501_02573_amd import binding
    return binding.lib


def declared_functions(headers=HEADERS):
    names = set()
    for path in headers:
        text = re.sub(r"/\*.*?\*/", "", open(path).read(), flags=re.S)
        names |= set(re.findall(r"\b(leet_attn_\w+)\s*\(", text))
    return sorted(names)


def test_header_declares_the_mandated_entry_points():
    names = declared_functions([HEADER])
    assert "leet_attn_forward" in names and "leet_attn_decode_step" in names
    assert len(names) >= 6
    # the measurement aids are declared apart from the attention boundary
    assert "leet_attn_forward_profile" not in names and "leet_attn_calibration_stream" not in names
    assert set(declared_functions()) == set(names) | {"leet_attn_forward_profile", "leet_attn_calibration_stream"}


def test_library_exports_every_declared_symbol(lib):
    from paper_2501_02573_amd import binding
    raw = ctypes.CDLL(LIB)
    for name in declared_functions():
        assert hasattr(raw, name), f"{name} declared in include/ but not exported"
        assert name in binding.EXPORTED_SYMBOLS
    assert set(binding.EXPORTED_SYMBOLS) == set(declared_functions())


def test_strerror_and_version(lib):
    from paper_2501_02573_amd import binding
    assert binding.strerror(0) == "ok"
    for st in (1, 2, 3, 4, 5, 6, 99):
        assert len(binding.strerror(st)) > 0
    assert re.fullmatch(r"\d+\.\d+\.\d+", binding.version())


def test_workspace_bytes_plan(lib):
    from paper_2501_02573_amd import binding as b
    # one segment -> no workspace
    assert b.workspace_bytes(1, 1, 64, 64, b.LEET_F32) == 0
    # with segments: one state per boundary, plus one per sequence for the copy of the entering state
    assert b.workspace_bytes(1, 1, 256, 64, b.LEET_F32) == (3 + 1) * 64 * 64 * 4  # fp32, short sequence: four segments of one chunk
    assert b.workspace_bytes(1, 1, 8192, 64, b.LEET_F32) == (63 + 1) * 64 * 64 * 4  # fp32, long sequence: segments of two chunks
    # fp32, long segments: the pre-pass computes its states on quarter-segments (3 boundaries x 4 + the copy)
    assert b.workspace_bytes(4, 16, 4096, 128, b.LEET_F32) == 4 * 16 * (12 + 1) * 128 * 128 * 4
    assert b.workspace_bytes(1, 1, 256, 64, b.LEET_BF16) == 0
    assert b.workspace_bytes(4, 16, 4096, 128, b.LEET_BF16, 1) == 0
    # s segments -> (s-1) boundary states of d*d floats per (b,h), and the entering-state copy
    assert b.workspace_bytes(4, 16, 4096, 128, b.LEET_BF16, 8) == 4 * 16 * (7 + 1) * 128 * 128 * 4
    assert b.workspace_bytes(1, 32, 32768, 128, b.LEET_BF16, 16) == 32 * (15 + 1) * 128 * 128 * 4
    # requests beyond the number of chunks are clamped: N=130 has 3 chunks
    assert b.workspace_bytes(1, 1, 130, 64, b.LEET_F32, 50) == (2 + 1) * 64 * 64 * 4
    # invalid shapes report 0
    assert b.workspace_bytes(1, 1, 256, 96, b.LEET_F32) == 0
    assert b.workspace_bytes(0, 1, 256, 64, b.LEET_F32) == 0


def test_bad_arguments_are_rejected_on_the_host(lib):
    """These return before any device call, so fake non-null pointers are never dereferenced."""
    from paper_2501_02573_amd import binding as b
    p = ctypes.c_void_p(0x1000)   # 16-byte aligned, never touched
    odd = ctypes.c_void_p(0x1004)
    fwd = lib.leet_attn_forward
    assert fwd(None, p, p, p, p, 1, 1, 64, 64, b.LEET_F32, None) == b.LEET_ERR_INVALID_ARG
    assert fwd(p, p, p, None, p, 1, 1, 64, 64, b.LEET_F32, None) == b.LEET_ERR_INVALID_ARG
    assert fwd(p, p, p, p, None, 1, 1, 64, 64, b.LEET_F32, None) == b.LEET_ERR_INVALID_ARG
    assert fwd(p, p, p, p, p, 0, 1, 64, 64, b.LEET_F32, None) == b.LEET_ERR_INVALID_ARG
    assert fwd(p, p, p, p, p, 1, 1, -5, 64, b.LEET_F32, None) == b.LEET_ERR_INVALID_ARG
    assert fwd(p, p, p, p, p, 1, 1, 64, 96, b.LEET_F32, None) == b.LEET_ERR_UNSUPPORTED
    assert fwd(p, p, p, p, p, 1, 1, 64, 64, 7, None) == b.LEET_ERR_UNSUPPORTED
    assert fwd(odd, p, p, p, p, 1, 1, 64, 64, b.LEET_F32, None) == b.LEET_ERR_INVALID_ARG
    assert fwd(p, p, p, p, p, 1 << 16, 1 << 16, 64, 64, b.LEET_F32, None) == b.LEET_ERR_TOO_LARGE
    dec = lib.leet_attn_decode_step
    assert dec(p, p, p, p, None, p, 1, 1, 64, None) == b.LEET_ERR_INVALID_ARG
    assert dec(p, p, p, p, p, p, 1, 0, 64, None) == b.LEET_ERR_INVALID_ARG
    assert dec(p, p, p, p, p, p, 1, 1, 32, None) == b.LEET_ERR_UNSUPPORTED
    assert lib.leet_attn_decode_step_ex(p, p, p, p, p, p, 1, 1, 64, 5, None) == b.LEET_ERR_UNSUPPORTED
    # no tokens: legal, q, k, v, out may be null, and with no state to write nothing touches a device
    assert fwd(None, None, None, p, None, 1, 1, 0, 64, b.LEET_F32, None) == b.LEET_OK
    assert fwd(None, None, None, None, None, 1, 1, 0, 64, b.LEET_F32, None) == b.LEET_ERR_INVALID_ARG   # gamma still required
    assert fwd(None, None, None, p, None, 1, 1, 0, 96, b.LEET_F32, None) == b.LEET_ERR_UNSUPPORTED
    assert lib.leet_attn_workspace_bytes(1, 1, 0, 64, b.LEET_F32, 0) == 0
    assert b.query_plan(4, 2, 0, 128, b.LEET_BF16) == (0, b.KERNEL_WIDE)
    ex = lib.leet_attn_forward_ex
    assert ex(None, None, None, p, None, p, p, None, 0, 0, 1, 1, 0, 64, b.LEET_F32, None) == b.LEET_OK   # state handed on in place
    assert ex(p, p, p, p, p, None, None, None, 0, -1, 1, 1, 64, 64, b.LEET_F32, None) == b.LEET_ERR_INVALID_ARG
    assert ex(p, p, p, p, p, odd, None, None, 0, 0, 1, 1, 64, 64, b.LEET_F32, None) == b.LEET_ERR_INVALID_ARG


def test_profile_entry_rejects_state_handed_on_in_place(lib):
    """The timing aid launches the walk several times; with state_out aliasing state_in the later
    launches would start from the wrong state, so it refuses (on the host, before any device call)."""
    from paper_2501_02573_amd import binding as b
    p = ctypes.c_void_p(0x1000)
    s = ctypes.c_void_p(0x2000)
    ms = (ctypes.c_float * 3)()
    prof = lib.leet_attn_forward_profile
    assert prof(p, p, p, p, p, s, s, None, 0, 0, 1, 1, 64, 64, b.LEET_F32, None, ms) == b.LEET_ERR_INVALID_ARG
    assert prof(p, p, p, p, p, s, s, None, 0, 0, 1, 1, 64, 64, b.LEET_F32, None, None) == b.LEET_ERR_INVALID_ARG


def test_kernel_choice_setter_and_plan_query(lib):
    from paper_2501_02573_amd import binding as b
    assert b.get_bf16_kernel() == b.KERNEL_AUTO
    try:
        # automatic choice: the cheapest (kernel, segment count) pair by the library's cost model
        assert b.query_plan(4, 16, 4096, 128, b.LEET_BF16) == (1, b.KERNEL_COLUMN_SPLIT)      # 256 workgroups, one kernel
        assert b.query_plan(1, 32, 32768, 128, b.LEET_BF16)[1] == b.KERNEL_WIDE              # inputs beyond the cache
        assert b.query_plan(16, 32, 4096, 128, b.LEET_BF16) == (1, b.KERNEL_WIDE)            # plenty of sequences
        assert b.query_plan(4, 16, 128, 128, b.LEET_BF16) == (1, b.KERNEL_WIDE)              # two chunks: too short
        assert b.query_plan(4, 16, 512, 128, b.LEET_BF16) == (1, b.KERNEL_COLUMN_SPLIT)
        assert b.query_plan(2, 16, 1024, 128, b.LEET_BF16) == (1, b.KERNEL_COLUMN_SPLIT)     # small job: launches dominate
        assert b.query_plan(2, 16, 4096, 128, b.LEET_BF16) == (8, b.KERNEL_WIDE)             # half the device, long
        assert b.query_plan(4, 18, 4096, 128, b.LEET_BF16)[1] == b.KERNEL_WIDE               # 288 workgroups: a second round
        assert b.query_plan(4, 15, 4096, 128, b.LEET_BF16) == (1, b.KERNEL_COLUMN_SPLIT)     # 240 workgroups, whole sequences
        # inputs beyond the cache: the two kernels measure within 1 % of each other here
        assert b.query_plan(4, 16, 16384, 128, b.LEET_BF16) in ((1, b.KERNEL_COLUMN_SPLIT), (4, b.KERNEL_WIDE))
        assert b.query_plan(8, 16, 16384, 64, b.LEET_BF16) == (1, b.KERNEL_COLUMN_SPLIT)     # d = 64: two slices a sequence
        assert b.query_plan(8, 16, 4096, 64, b.LEET_BF16) == (1, b.KERNEL_COLUMN_SPLIT)
        assert b.query_plan(4, 16, 4096, 128, b.LEET_F32)[1] == b.KERNEL_WIDE                # 16-bit inputs only
        assert b.query_plan(4, 16, 4096, 128, b.LEET_F16) == (1, b.KERNEL_COLUMN_SPLIT)         # both 16-bit types
        # a lone sequence: many short segments of the column-split kernel
        nseg, kern = b.query_plan(1, 1, 4096, 128, b.LEET_BF16)
        assert kern == b.KERNEL_COLUMN_SPLIT and 8 <= nseg <= 16
        # a caller's segment count is kept; the kernel is still chosen
        assert b.query_plan(4, 16, 4096, 128, b.LEET_BF16, 4) == (4, b.KERNEL_WIDE)
        assert b.query_plan(1, 1, 4096, 128, b.LEET_BF16, 8) == (8, b.KERNEL_COLUMN_SPLIT)
        assert b.workspace_bytes(4, 16, 4096, 128, b.LEET_BF16) == 0
        b.set_bf16_kernel(b.KERNEL_COLUMN_SPLIT)
        assert b.get_bf16_kernel() == b.KERNEL_COLUMN_SPLIT
        assert b.query_plan(1, 32, 32768, 128, b.LEET_BF16)[1] == b.KERNEL_COLUMN_SPLIT
        assert b.query_plan(4, 16, 128, 128, b.LEET_BF16) == (1, b.KERNEL_COLUMN_SPLIT)      # forced: any length
        b.set_bf16_kernel(b.KERNEL_WIDE)
        assert b.query_plan(4, 16, 4096, 128, b.LEET_BF16) == (4, b.KERNEL_WIDE)
        # four segments for the walk, boundary states on half-segments for the pre-pass and the scan
        assert b.workspace_bytes(4, 16, 4096, 128, b.LEET_BF16) == 4 * 16 * (6 + 1) * 128 * 128 * 4
        with pytest.raises(b.LeetAttnError):
            b.set_bf16_kernel(7)
        assert b.get_bf16_kernel() == b.KERNEL_WIDE
        with pytest.raises(b.LeetAttnError):
            b.query_plan(1, 1, 64, 96, b.LEET_BF16)
    finally:
        b.set_bf16_kernel(b.KERNEL_AUTO)


def test_planner_against_measured_sweep(lib):
    """The planner's pick is within 12 % of the fastest measured (kernel, segment count) pair on every
    shape of the tabulated sweep (the worst of 262 is 8.3 %), and within 1 % on average (0.24 %)."""
    import json
    from paper_2501_02573_amd import binding as b
    table = json.load(open(os.path.join(ROOT, "profiles", "plan_sweep.json")))
    ratios = []
    for key, runs in table.items():
        if key.startswith("_"):
            continue
        d, bh, n = (int(x) for x in key.split(","))
        if d == 256:     # rank 128, value width 256
            nseg, kern = b.query_plan_rd(1, bh, n, 128, 256, b.LEET_BF16)
        else:
            nseg, kern = b.query_plan(1, bh, n, d, b.LEET_BF16)
        label = ("c" if kern == b.KERNEL_COLUMN_SPLIT else "w") + str(nseg)
        if label not in runs:      # a rounded segment count that the sweep did not time
            continue
        ratio = runs[label] / min(runs.values())
        assert ratio <= 1.12, (key, label, runs[label], min(runs.values()))
        ratios.append(ratio)
    assert len(ratios) >= 200
    assert sum(ratios) / len(ratios) <= 1.01


def test_planner_invariants_on_random_shapes(lib):
    """Whatever the cost model prefers, a plan is well-formed: between 1 and ceil(N/64) segments,
    a caller's segment count honoured up to rounding, and a workspace of one state per segment
    boundary (two on the wide 16-bit and fp32 paths when they compute them on half-segments)."""
    import random
    from paper_2501_02573_amd import binding as b
    rng = random.Random(7)
    for _ in range(400):
        d = rng.choice((64, 128))
        dtype = rng.choice((b.LEET_F32, b.LEET_BF16, b.LEET_F16))
        B, H = rng.randint(1, 6), rng.randint(1, 48)
        N = rng.choice((1, 63, 64, 65, 500, 1000, 4096, 5000, 33000, 100000, rng.randint(1, 200000)))
        segs = rng.choice((0, 0, 0, 1, 2, 3, 5, 8, 100))
        nchunks = -(-N // 64)
        nseg, kern = b.query_plan(B, H, N, d, dtype, segs)
        assert 1 <= nseg <= nchunks, (B, H, N, d, dtype, segs, nseg)
        if segs:
            want = min(segs, nchunks)
            seg_chunks = -(-nchunks // want)
            assert nseg == -(-nchunks // seg_chunks)
        if dtype == b.LEET_F32:
            assert kern == b.KERNEL_WIDE
        ws = b.workspace_bytes(B, H, N, d, dtype, segs)
        state = B * H * d * d * 4
        assert ws % state == 0
        slots = ws // state
        extra = 1 if nseg > 1 else 0    # the copy of the entering state
        if kern == b.KERNEL_COLUMN_SPLIT:
            assert slots == nseg - 1 + extra
        elif dtype == b.LEET_F32:      # the fp32 pre-pass runs on segments 1, 2, 4 or 8 times finer than the walk's
            assert slots in [m * (nseg - 1) + extra for m in (1, 2, 4, 8)]
        else:
            assert slots in (nseg - 1 + extra, 2 * (nseg - 1) + extra)


def test_binding_rejects_cpu_tensors(lib):
    import torch
    from paper_2501_02573_amd import binding as b
    q = torch.zeros(1, 1, 64, 64)
    g = torch.ones(1)
    with pytest.raises(ValueError):
        b.leet_attn_forward(q, q, q, g, torch.empty_like(q))


def test_decode_store_knob(lib):
    from paper_2501_02573_amd import binding as b
    assert b.get_decode_store() == b.DECODE_STORE_AUTO
    try:
        for mode in (b.DECODE_STORE_CACHED, b.DECODE_STORE_STREAM, b.DECODE_STORE_AUTO):
            b.set_decode_store(mode)
            assert b.get_decode_store() == mode
        with pytest.raises(b.LeetAttnError):
            b.set_decode_store(5)
    finally:
        b.set_decode_store(b.DECODE_STORE_AUTO)


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as strict C99 and declare every exported symbol."""
    import subprocess
    from paper_2501_02573_amd import binding as b
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "use_header.c"
    calls = "\n".join(f"    (void)&{name};" for name in b.EXPORTED_SYMBOLS)
    src.write_text('#include "leet_attn.h"\n#include "leet_attn_bench.h"\nint main(void) {\n' + calls + "\n    return 0;\n}\n")
    res = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only",
                          "-I", os.path.join(root, "include"), str(src)], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr


def test_per_call_choices_match_the_setters(lib):
    """The _v3 queries take the kernel choice as an argument: same answers as under the setter, and
    independent of what the process-wide default is set to meanwhile."""
    from paper_2501_02573_amd import binding as b
    shapes = [(4, 16, 4096, 128, 128), (1, 32, 32768, 128, 128), (1, 1, 4096, 128, 128), (2, 3, 777, 64, 64),
              (1, 32, 2048, 128, 256)]
    try:
        want = {}
        for choice in (b.KERNEL_WIDE, b.KERNEL_COLUMN_SPLIT, b.KERNEL_AUTO):
            b.set_bf16_kernel(choice)
            for sh in shapes:
                want[(choice, sh)] = (b.query_plan_rd(*sh[:3], sh[3], sh[4], b.LEET_BF16),
                                      b.workspace_bytes_rd(*sh[:3], sh[3], sh[4], b.LEET_BF16))
        for default in (b.KERNEL_WIDE, b.KERNEL_COLUMN_SPLIT, b.KERNEL_AUTO):
            b.set_bf16_kernel(default)
            for (choice, sh), (plan, ws) in want.items():
                assert b.query_plan_v3(*sh[:3], sh[3], sh[4], b.LEET_BF16, 0, choice) == plan
                assert b.workspace_bytes_v3(*sh[:3], sh[3], sh[4], b.LEET_BF16, 0, choice) == ws
            for sh in shapes:   # LEET_CHOICE_DEFAULT follows the setter
                assert b.query_plan_v3(*sh[:3], sh[3], sh[4], b.LEET_BF16) == want[(default, sh)][0]
        with pytest.raises(b.LeetAttnError):
            b.query_plan_v3(1, 1, 4096, 128, 128, b.LEET_BF16, 0, 9)
        assert b.workspace_bytes_v3(1, 1, 4096, 128, 128, b.LEET_BF16, 0, 9) == 0
    finally:
        b.set_bf16_kernel(b.KERNEL_AUTO)
    p = ctypes.c_void_p(0x1000)
    assert lib.leet_attn_decode_step_v3(p, p, p, p, p, p, 1, 1, 64, 64, b.LEET_BF16, 0, 7, None) == b.LEET_ERR_INVALID_ARG
    assert lib.leet_attn_forward_v3(p, p, p, p, p, None, None, None, 0, 0, 7, 1, 1, 64, 64, 64, b.LEET_BF16, b.LEET_F32,
                                    0, None) == b.LEET_ERR_INVALID_ARG


def test_static_scratch_entry_point_limits(lib):
    """The entry point that allocates nothing refuses, on the host, plans whose segment states exceed
    its static scratch, and takes the same argument checks as leet_attn_forward_ex."""
    from paper_2501_02573_amd import binding as b
    cap = b.static_scratch_bytes()
    assert cap == 32 << 20
    p = ctypes.c_void_p(0x1000)
    st = lib.leet_attn_forward_static
    # the long-context benchmark shape fits under the library's own plan
    assert 0 < b.workspace_bytes(1, 32, 32768, 128, b.LEET_BF16) <= cap
    # 64 sequences cut into 16 segments: 64 * 16 states of 64 KiB = 64 MiB
    assert b.workspace_bytes(4, 16, 8192, 128, b.LEET_BF16, 16) > cap
    assert st(p, p, p, p, p, None, None, 16, 4, 16, 8192, 128, b.LEET_BF16, None) == b.LEET_ERR_SCRATCH_LIMIT
    assert st(None, p, p, p, p, None, None, 0, 1, 1, 64, 64, b.LEET_F32, None) == b.LEET_ERR_INVALID_ARG
    assert st(p, p, p, p, p, None, None, 0, 1, 1, 64, 96, b.LEET_F32, None) == b.LEET_ERR_UNSUPPORTED
    assert st(p, p, p, p, p, None, None, 0, 1, 1, 64, 64, b.LEET_F16, None) == b.LEET_ERR_UNSUPPORTED
    assert "32 MiB" in b.strerror(b.LEET_ERR_SCRATCH_LIMIT)
