"""ctypes binding of libleet_attn.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU, checks shapes,
dtypes and contiguity on the host, and passes raw device pointers plus the current
torch stream to the C ABI declared in ``include/leet_attn.h``.  No arithmetic of the
operator happens here, and there is no fallback: if the native library is missing the
import of this module fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libleet_attn.so")

LEET_F32, LEET_BF16, LEET_F16 = 0, 1, 2
LEET_MASK_DECAY, LEET_MASK_CAUSAL = 0, 1
LEET_OK, LEET_ERR_INVALID_ARG, LEET_ERR_UNSUPPORTED, LEET_ERR_LAUNCH, LEET_ERR_TOO_LARGE = 0, 1, 2, 3, 4
LEET_ERR_CAPTURE, LEET_ERR_SCRATCH_LIMIT = 5, 6
LEET_CHOICE_DEFAULT = -1

EXPORTED_SYMBOLS = (
    "leet_attn_forward",
    "leet_attn_decode_step",
    "leet_attn_decode_step_ex",
    "leet_attn_forward_ex",
    "leet_attn_forward_v2",
    "leet_attn_decode_step_v2",
    "leet_attn_forward_recurrent",
    "leet_attn_forward_rd",
    "leet_attn_forward_recurrent_rd",
    "leet_attn_forward_fleet",
    "leet_attn_decode_step_rd",
    "leet_attn_workspace_bytes_rd",
    "leet_attn_forward_v3",
    "leet_attn_workspace_bytes_v3",
    "leet_attn_query_plan_v3",
    "leet_attn_decode_step_v3",
    "leet_attn_forward_static",
    "leet_attn_static_scratch_bytes",
    "leet_attn_forward_profile",
    "leet_attn_calibration_stream",
    "leet_attn_set_bf16_kernel",
    "leet_attn_get_bf16_kernel",
    "leet_attn_query_plan",
    "leet_attn_query_plan_rd",
    "leet_attn_set_decode_store",
    "leet_attn_get_decode_store",
    "leet_attn_workspace_bytes",
    "leet_attn_release_workspace",
    "leet_attn_strerror",
    "leet_attn_version",
)


class LeetAttnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status}: {strerror(status)}")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2501_02573_amd.build` "
            "(there is no CPU or PyTorch fallback for this library)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.leet_attn_forward.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, vp]
    lib.leet_attn_forward.restype = i
    lib.leet_attn_forward_ex.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, sz, i, i, i, i, i, i, vp]
    lib.leet_attn_forward_ex.restype = i
    lib.leet_attn_forward_v2.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, sz, i, i, i, i, i, i, i, i, vp]
    lib.leet_attn_forward_v2.restype = i
    lib.leet_attn_decode_step_v2.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, i, vp]
    lib.leet_attn_decode_step_v2.restype = i
    lib.leet_attn_forward_recurrent.argtypes = [vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, vp]
    lib.leet_attn_forward_recurrent.restype = i
    lib.leet_attn_forward_rd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, sz, i, i, i, i, i, i, i, i, i, vp]
    lib.leet_attn_forward_rd.restype = i
    lib.leet_attn_forward_recurrent_rd.argtypes = [vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, vp]
    lib.leet_attn_forward_recurrent_rd.restype = i
    lib.leet_attn_forward_fleet.argtypes = [vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, vp]
    lib.leet_attn_forward_fleet.restype = i
    lib.leet_attn_decode_step_rd.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, vp]
    lib.leet_attn_decode_step_rd.restype = i
    lib.leet_attn_workspace_bytes_rd.argtypes = [i, i, i, i, i, i, i]
    lib.leet_attn_workspace_bytes_rd.restype = sz
    lib.leet_attn_forward_v3.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, sz, i, i, i, i, i, i, i, i, i, i, vp]
    lib.leet_attn_forward_v3.restype = i
    lib.leet_attn_workspace_bytes_v3.argtypes = [i, i, i, i, i, i, i, i]
    lib.leet_attn_workspace_bytes_v3.restype = sz
    lib.leet_attn_query_plan_v3.argtypes = [i, i, i, i, i, i, i, i, ctypes.POINTER(i), ctypes.POINTER(i)]
    lib.leet_attn_query_plan_v3.restype = i
    lib.leet_attn_decode_step_v3.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, vp]
    lib.leet_attn_decode_step_v3.restype = i
    lib.leet_attn_forward_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, vp]
    lib.leet_attn_forward_static.restype = i
    lib.leet_attn_static_scratch_bytes.argtypes = []
    lib.leet_attn_static_scratch_bytes.restype = sz
    lib.leet_attn_forward_profile.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, sz, i, i, i, i, i, i, vp,
                                              ctypes.POINTER(ctypes.c_float)]
    lib.leet_attn_forward_profile.restype = i
    lib.leet_attn_calibration_stream.argtypes = [i, vp, vp, sz, i, vp]
    lib.leet_attn_calibration_stream.restype = i
    lib.leet_attn_decode_step.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, vp]
    lib.leet_attn_decode_step.restype = i
    lib.leet_attn_decode_step_ex.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, vp]
    lib.leet_attn_decode_step_ex.restype = i
    lib.leet_attn_workspace_bytes.argtypes = [i, i, i, i, i, i]
    lib.leet_attn_workspace_bytes.restype = sz
    lib.leet_attn_release_workspace.argtypes = []
    lib.leet_attn_release_workspace.restype = i
    lib.leet_attn_set_bf16_kernel.argtypes = [i]
    lib.leet_attn_set_bf16_kernel.restype = i
    lib.leet_attn_get_bf16_kernel.argtypes = []
    lib.leet_attn_get_bf16_kernel.restype = i
    lib.leet_attn_query_plan.argtypes = [i, i, i, i, i, i, ctypes.POINTER(i), ctypes.POINTER(i)]
    lib.leet_attn_query_plan.restype = i
    lib.leet_attn_query_plan_rd.argtypes = [i, i, i, i, i, i, i, ctypes.POINTER(i), ctypes.POINTER(i)]
    lib.leet_attn_query_plan_rd.restype = i
    lib.leet_attn_set_decode_store.argtypes = [i]
    lib.leet_attn_set_decode_store.restype = i
    lib.leet_attn_get_decode_store.argtypes = []
    lib.leet_attn_get_decode_store.restype = i
    lib.leet_attn_strerror.argtypes = [i]
    lib.leet_attn_strerror.restype = ctypes.c_char_p
    lib.leet_attn_version.argtypes = []
    lib.leet_attn_version.restype = ctypes.c_char_p
    return lib


lib = _load()


def strerror(status: int) -> str:
    return lib.leet_attn_strerror(int(status)).decode()


def version() -> str:
    return lib.leet_attn_version().decode()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return LEET_F32
    if t.dtype == torch.bfloat16:
        return LEET_BF16
    if t.dtype == torch.float16:
        return LEET_F16
    raise TypeError(f"unsupported dtype {t.dtype}: q, k, v must be float32, bfloat16 or float16")


def _check_dev(*tensors: Optional[torch.Tensor]) -> torch.device:
    dev = None
    for t in tensors:
        if t is None:
            continue
        if not t.is_cuda:
            raise ValueError("all tensors must be GPU tensors")
        if not t.is_contiguous():
            raise ValueError("all tensors must be contiguous")
        if dev is None:
            dev = t.device
        elif t.device != dev:
            raise ValueError("all tensors must be on one device")
    return dev


def _stream_ptr(dev: torch.device) -> int:
    return torch.cuda.current_stream(dev).cuda_stream


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


KERNEL_WIDE, KERNEL_COLUMN_SPLIT, KERNEL_AUTO = 0, 1, 2


def set_bf16_kernel(which: int) -> None:
    st = lib.leet_attn_set_bf16_kernel(int(which))
    if st != LEET_OK:
        raise LeetAttnError(st, "leet_attn_set_bf16_kernel")


def get_bf16_kernel() -> int:
    return int(lib.leet_attn_get_bf16_kernel())


DECODE_STORE_AUTO, DECODE_STORE_CACHED, DECODE_STORE_STREAM = 0, 1, 2


def set_decode_store(mode: int) -> None:
    st = lib.leet_attn_set_decode_store(int(mode))
    if st != LEET_OK:
        raise LeetAttnError(st, "leet_attn_set_decode_store")


def get_decode_store() -> int:
    return int(lib.leet_attn_get_decode_store())


def query_plan(B: int, H: int, N: int, d: int, dtype: int, segments: int = 0):
    """(segments per sequence, kernel) the library would use for this shape (host-only query)."""
    nseg, kern = ctypes.c_int(0), ctypes.c_int(0)
    st = lib.leet_attn_query_plan(B, H, N, d, dtype, segments, ctypes.byref(nseg), ctypes.byref(kern))
    if st != LEET_OK:
        raise LeetAttnError(st, "leet_attn_query_plan")
    return nseg.value, kern.value


def query_plan_rd(B: int, H: int, N: int, r: int, dv: int, dtype: int, segments: int = 0):
    """``query_plan`` for rank r and value width dv given separately."""
    nseg, kern = ctypes.c_int(0), ctypes.c_int(0)
    st = lib.leet_attn_query_plan_rd(B, H, N, r, dv, dtype, segments, ctypes.byref(nseg), ctypes.byref(kern))
    if st != LEET_OK:
        raise LeetAttnError(st, "leet_attn_query_plan_rd")
    return nseg.value, kern.value


def workspace_bytes(B: int, H: int, N: int, d: int, dtype: int, segments: int = 0) -> int:
    return int(lib.leet_attn_workspace_bytes(B, H, N, d, dtype, segments))


def release_workspace() -> None:
    st = lib.leet_attn_release_workspace()
    if st != LEET_OK:
        raise LeetAttnError(st, "leet_attn_release_workspace")


def _check_forward(q, k, v, gamma, out, any_out_dtype: bool = False):
    if q.dim() != 4 or q.shape != k.shape or q.shape != v.shape:
        raise ValueError("q, k, v must share one [B, H, N, d] shape")
    if k.dtype != q.dtype or v.dtype != q.dtype:
        raise TypeError("q, k, v must share one dtype")
    B, H, N, d = q.shape
    if gamma is not None and (gamma.dtype != torch.float32 or gamma.numel() != H):
        raise ValueError("gamma must be float32 with one value per head")
    if out.shape != q.shape or (out.dtype != torch.float32 and not any_out_dtype):
        raise ValueError("out must be float32 [B, H, N, d]")
    return B, H, N, d


def leet_attn_forward(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, gamma: torch.Tensor,
                      out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Chunked prefill with zero initial state; returns fp32 ``out`` [B, H, N, d]."""
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    B, H, N, d = _check_forward(q, k, v, gamma, out)
    dev = _check_dev(q, k, v, gamma, out)
    with torch.cuda.device(dev):
        st = lib.leet_attn_forward(_ptr(q), _ptr(k), _ptr(v), _ptr(gamma), _ptr(out), B, H, N, d,
                                   _dtype_code(q), ctypes.c_void_p(_stream_ptr(dev)))
    if st != LEET_OK:
        raise LeetAttnError(st, "leet_attn_forward")
    return out


def leet_attn_forward_ex(q, k, v, gamma, out: Optional[torch.Tensor] = None,
                         state_in: Optional[torch.Tensor] = None,
                         state_out: Optional[torch.Tensor] = None,
                         workspace: Optional[torch.Tensor] = None, segments: int = 0) -> torch.Tensor:
    """Chunked prefill with state hand-off and optional caller-owned workspace."""
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    B, H, N, d = _check_forward(q, k, v, gamma, out)
    for name, s in (("state_in", state_in), ("state_out", state_out)):
        if s is not None and (s.dtype != torch.float32 or tuple(s.shape) != (B, H, d, d)):
            raise ValueError(f"{name} must be float32 [B, H, d, d]")
    ws_bytes = 0
    if workspace is not None:
        if workspace.dtype != torch.uint8:
            raise TypeError("workspace must be a uint8 tensor")
        ws_bytes = workspace.numel()
    dev = _check_dev(q, k, v, gamma, out, state_in, state_out, workspace)
    with torch.cuda.device(dev):
        st = lib.leet_attn_forward_ex(_ptr(q), _ptr(k), _ptr(v), _ptr(gamma), _ptr(out), _ptr(state_in),
                                      _ptr(state_out), _ptr(workspace), ws_bytes, int(segments),
                                      B, H, N, d, _dtype_code(q), ctypes.c_void_p(_stream_ptr(dev)))
    if st != LEET_OK:
        raise LeetAttnError(st, "leet_attn_forward_ex")
    return out


def leet_attn_forward_v2(q, k, v, gamma: Optional[torch.Tensor], out: Optional[torch.Tensor] = None,
                         state_in: Optional[torch.Tensor] = None,
                         state_out: Optional[torch.Tensor] = None,
                         workspace: Optional[torch.Tensor] = None, segments: int = 0,
                         out_dtype: Optional[torch.dtype] = None,
                         mask: int = LEET_MASK_DECAY) -> torch.Tensor:
    """Chunked prefill with every option: fp16 inputs, output in the input type, 0/1 causal mask.

    ``out_dtype`` (used when ``out`` is None) defaults to float32; ``gamma`` may be None with
    ``mask=LEET_MASK_CAUSAL``.  Unsupported combinations are reported by the library.
    """
    if out is None:
        out = torch.empty(q.shape, dtype=out_dtype or torch.float32, device=q.device)
    B, H, N, d = _check_forward(q, k, v, gamma, out, any_out_dtype=True)
    for name, s in (("state_in", state_in), ("state_out", state_out)):
        if s is not None and (s.dtype != torch.float32 or tuple(s.shape) != (B, H, d, d)):
            raise ValueError(f"{name} must be float32 [B, H, d, d]")
    ws_bytes = 0
    if workspace is not None:
        if workspace.dtype != torch.uint8:
            raise TypeError("workspace must be a uint8 tensor")
        ws_bytes = workspace.numel()
    dev = _check_dev(q, k, v, gamma, out, state_in, state_out, workspace)
    with torch.cuda.device(dev):
        st = lib.leet_attn_forward_v2(_ptr(q), _ptr(k), _ptr(v), _ptr(gamma), _ptr(out), _ptr(state_in),
                                      _ptr(state_out), _ptr(workspace), ws_bytes, int(segments),
                                      B, H, N, d, _dtype_code(q), _dtype_code(out), int(mask),
                                      ctypes.c_void_p(_stream_ptr(dev)))
    if st != LEET_OK:
        raise LeetAttnError(st, "leet_attn_forward_v2")
    return out


def leet_attn_forward_recurrent(q, k, v, gamma: Optional[torch.Tensor], out: Optional[torch.Tensor] = None,
                                state_in: Optional[torch.Tensor] = None,
                                state_out: Optional[torch.Tensor] = None,
                                mask: int = LEET_MASK_DECAY) -> torch.Tensor:
    """Row-based (token-by-token) prefill on the GPU: the comparison point for the chunked path."""
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    B, H, N, d = _check_forward(q, k, v, gamma, out)
    for name, s in (("state_in", state_in), ("state_out", state_out)):
        if s is not None and (s.dtype != torch.float32 or tuple(s.shape) != (B, H, d, d)):
            raise ValueError(f"{name} must be float32 [B, H, d, d]")
    dev = _check_dev(q, k, v, gamma, out, state_in, state_out)
    with torch.cuda.device(dev):
        st = lib.leet_attn_forward_recurrent(_ptr(q), _ptr(k), _ptr(v), _ptr(gamma), _ptr(out), _ptr(state_in),
                                             _ptr(state_out), B, H, N, d, _dtype_code(q), int(mask),
                                             ctypes.c_void_p(_stream_ptr(dev)))
    if st != LEET_OK:
        raise LeetAttnError(st, "leet_attn_forward_recurrent")
    return out


def leet_attn_forward_profile(q, k, v, gamma, out: Optional[torch.Tensor] = None, segments: int = 0):
    """One prefill with per-kernel HIP-event timing; returns (out, [pre-pass ms, scan ms, walk ms])."""
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    B, H, N, d = _check_forward(q, k, v, gamma, out)
    dev = _check_dev(q, k, v, gamma, out)
    ms = (ctypes.c_float * 3)()
    with torch.cuda.device(dev):
        st = lib.leet_attn_forward_profile(_ptr(q), _ptr(k), _ptr(v), _ptr(gamma), _ptr(out), None, None,
                                           None, 0, int(segments), B, H, N, d, _dtype_code(q),
                                           ctypes.c_void_p(_stream_ptr(dev)), ms)
    if st != LEET_OK:
        raise LeetAttnError(st, "leet_attn_forward_profile")
    return out, [float(x) for x in ms]


def calibration_stream(mode: str, src: Optional[torch.Tensor], dst: torch.Tensor, nbytes: int,
                       workgroups: int = 4096) -> None:
    """Launches the plain copy / read / fill kernel over ``nbytes`` (measurement aid)."""
    code = {"copy": 0, "read": 1, "fill": 2, "copy_nt": 3, "fill_nt": 4}[mode]
    dev = _check_dev(src, dst)
    with torch.cuda.device(dev):
        st = lib.leet_attn_calibration_stream(code, _ptr(src), _ptr(dst), int(nbytes), int(workgroups),
                                              ctypes.c_void_p(_stream_ptr(dev)))
    if st != LEET_OK:
        raise LeetAttnError(st, "leet_attn_calibration_stream")


def _check_decode(q, k, v, gamma, state, out):
    if q.dim() != 3 or q.shape != k.shape or q.shape != v.shape:
        raise ValueError("q, k, v must share one [B, H, d] shape")
    if k.dtype != q.dtype or v.dtype != q.dtype:
        raise TypeError("q, k, v must share one dtype")
    B, H, d = q.shape
    if gamma is not None and (gamma.dtype != torch.float32 or gamma.numel() != H):
        raise ValueError("gamma must be float32 with one value per head")
    if state.dtype != torch.float32 or tuple(state.shape) != (B, H, d, d):
        raise ValueError("state must be float32 [B, H, d, d]")
    if out.dtype != torch.float32 or tuple(out.shape) != (B, H, d):
        raise ValueError("out must be float32 [B, H, d]")
    return B, H, d


def leet_attn_decode_step(q, k, v, gamma, state, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """One decode step with bf16 q, k, v: ``state`` is updated in place; returns fp32 ``out`` [B, H, d]."""
    if q.dtype != torch.bfloat16:
        raise TypeError("leet_attn_decode_step takes bfloat16 q, k, v (use leet_attn_decode_step_ex for float32)")
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    B, H, d = _check_decode(q, k, v, gamma, state, out)
    dev = _check_dev(q, k, v, gamma, state, out)
    with torch.cuda.device(dev):
        st = lib.leet_attn_decode_step(_ptr(q), _ptr(k), _ptr(v), _ptr(gamma), _ptr(state), _ptr(out),
                                       B, H, d, ctypes.c_void_p(_stream_ptr(dev)))
    if st != LEET_OK:
        raise LeetAttnError(st, "leet_attn_decode_step")
    return out


def leet_attn_decode_step_ex(q, k, v, gamma, state, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """One decode step with float32 or bfloat16 q, k, v."""
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    B, H, d = _check_decode(q, k, v, gamma, state, out)
    dev = _check_dev(q, k, v, gamma, state, out)
    with torch.cuda.device(dev):
        st = lib.leet_attn_decode_step_ex(_ptr(q), _ptr(k), _ptr(v), _ptr(gamma), _ptr(state), _ptr(out),
                                          B, H, d, _dtype_code(q), ctypes.c_void_p(_stream_ptr(dev)))
    if st != LEET_OK:
        raise LeetAttnError(st, "leet_attn_decode_step_ex")
    return out


def leet_attn_decode_step_v2(q, k, v, gamma: Optional[torch.Tensor], state, out: Optional[torch.Tensor] = None,
                             mask: int = LEET_MASK_DECAY) -> torch.Tensor:
    """One decode step with float32, bfloat16 or float16 q, k, v and either mask."""
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    B, H, d = _check_decode(q, k, v, gamma, state, out)
    dev = _check_dev(q, k, v, gamma, state, out)
    with torch.cuda.device(dev):
        st = lib.leet_attn_decode_step_v2(_ptr(q), _ptr(k), _ptr(v), _ptr(gamma), _ptr(state), _ptr(out),
                                          B, H, d, _dtype_code(q), int(mask), ctypes.c_void_p(_stream_ptr(dev)))
    if st != LEET_OK:
        raise LeetAttnError(st, "leet_attn_decode_step_v2")
    return out


# ---------------------------------------------------------------- rank r different from the value width dv
def workspace_bytes_rd(B: int, H: int, N: int, r: int, dv: int, dtype: int, segments: int = 0) -> int:
    return int(lib.leet_attn_workspace_bytes_rd(B, H, N, r, dv, dtype, segments))


def _check_rd(q, k, v, gamma, out, any_out_dtype):
    if q.dim() != 4 or q.shape != k.shape or v.dim() != 4 or q.shape[:3] != v.shape[:3]:
        raise ValueError("q, k must share one [B, H, N, r] shape and v be [B, H, N, dv]")
    if k.dtype != q.dtype or v.dtype != q.dtype:
        raise TypeError("q, k, v must share one dtype")
    B, H, N, r = q.shape
    dv = v.shape[3]
    if gamma is not None and (gamma.dtype != torch.float32 or gamma.numel() != H):
        raise ValueError("gamma must be float32 with one value per head")
    if out.shape != v.shape or (out.dtype != torch.float32 and not any_out_dtype):
        raise ValueError("out must be [B, H, N, dv]" + ("" if any_out_dtype else " float32"))
    return B, H, N, r, dv


def _check_states_rd(B, H, r, dv, **states):
    for name, s in states.items():
        if s is not None and (s.dtype != torch.float32 or tuple(s.shape) != (B, H, r, dv)):
            raise ValueError(f"{name} must be float32 [B, H, r, dv]")


def leet_attn_forward_rd(q, k, v, gamma: Optional[torch.Tensor], out: Optional[torch.Tensor] = None,
                         state_in: Optional[torch.Tensor] = None, state_out: Optional[torch.Tensor] = None,
                         workspace: Optional[torch.Tensor] = None, segments: int = 0,
                         out_dtype: Optional[torch.dtype] = None, mask: int = LEET_MASK_DECAY) -> torch.Tensor:
    """Chunked prefill with q, k of width r and v, out of width dv; states are [B, H, r, dv]."""
    if out is None:
        out = torch.empty(v.shape, dtype=out_dtype or torch.float32, device=v.device)
    B, H, N, r, dv = _check_rd(q, k, v, gamma, out, True)
    _check_states_rd(B, H, r, dv, state_in=state_in, state_out=state_out)
    ws_bytes = 0
    if workspace is not None:
        if workspace.dtype != torch.uint8:
            raise TypeError("workspace must be a uint8 tensor")
        ws_bytes = workspace.numel()
    dev = _check_dev(q, k, v, gamma, out, state_in, state_out, workspace)
    with torch.cuda.device(dev):
        st = lib.leet_attn_forward_rd(_ptr(q), _ptr(k), _ptr(v), _ptr(gamma), _ptr(out), _ptr(state_in),
                                      _ptr(state_out), _ptr(workspace), ws_bytes, int(segments),
                                      B, H, N, r, dv, _dtype_code(q), _dtype_code(out), int(mask),
                                      ctypes.c_void_p(_stream_ptr(dev)))
    if st != LEET_OK:
        raise LeetAttnError(st, "leet_attn_forward_rd")
    return out


def leet_attn_forward_v3(q, k, v, gamma: Optional[torch.Tensor], out: Optional[torch.Tensor] = None,
                         state_in: Optional[torch.Tensor] = None, state_out: Optional[torch.Tensor] = None,
                         workspace: Optional[torch.Tensor] = None, segments: int = 0,
                         kernel: int = LEET_CHOICE_DEFAULT,
                         out_dtype: Optional[torch.dtype] = None, mask: int = LEET_MASK_DECAY) -> torch.Tensor:
    """``leet_attn_forward_rd`` with the kernel choice given per call."""
    if out is None:
        out = torch.empty(v.shape, dtype=out_dtype or torch.float32, device=v.device)
    B, H, N, r, dv = _check_rd(q, k, v, gamma, out, True)
    _check_states_rd(B, H, r, dv, state_in=state_in, state_out=state_out)
    ws_bytes = 0
    if workspace is not None:
        if workspace.dtype != torch.uint8:
            raise TypeError("workspace must be a uint8 tensor")
        ws_bytes = workspace.numel()
    dev = _check_dev(q, k, v, gamma, out, state_in, state_out, workspace)
    with torch.cuda.device(dev):
        st = lib.leet_attn_forward_v3(_ptr(q), _ptr(k), _ptr(v), _ptr(gamma), _ptr(out), _ptr(state_in),
                                      _ptr(state_out), _ptr(workspace), ws_bytes, int(segments), int(kernel),
                                      B, H, N, r, dv, _dtype_code(q), _dtype_code(out), int(mask),
                                      ctypes.c_void_p(_stream_ptr(dev)))
    if st != LEET_OK:
        raise LeetAttnError(st, "leet_attn_forward_v3")
    return out


class PreparedForward:
    """``leet_attn_forward_v3`` with the argument checks and the marshalling done once.

    For a serving loop that calls the library again and again on the same buffers (contents may
    change, addresses and shapes may not): calling the object makes one ctypes call into
    ``leet_attn_forward_v3`` on the device's current stream (or on ``stream``, a raw stream handle,
    if one was given) and nothing else.  The object keeps the tensors alive."""

    def __init__(self, q, k, v, gamma: Optional[torch.Tensor], out: torch.Tensor,
                 state_in: Optional[torch.Tensor] = None, state_out: Optional[torch.Tensor] = None,
                 workspace: Optional[torch.Tensor] = None, segments: int = 0,
                 kernel: int = LEET_CHOICE_DEFAULT, mask: int = LEET_MASK_DECAY, stream: Optional[int] = None):
        B, H, N, r, dv = _check_rd(q, k, v, gamma, out, True)
        _check_states_rd(B, H, r, dv, state_in=state_in, state_out=state_out)
        ws_bytes = 0
        if workspace is not None:
            if workspace.dtype != torch.uint8:
                raise TypeError("workspace must be a uint8 tensor")
            ws_bytes = workspace.numel()
        self._dev = _check_dev(q, k, v, gamma, out, state_in, state_out, workspace)
        self._keep = (q, k, v, gamma, out, state_in, state_out, workspace)
        self._args = (_ptr(q), _ptr(k), _ptr(v), _ptr(gamma), _ptr(out), _ptr(state_in), _ptr(state_out),
                      _ptr(workspace), ws_bytes, int(segments), int(kernel), B, H, N, r, dv,
                      _dtype_code(q), _dtype_code(out), int(mask))
        self._stream = None if stream is None else ctypes.c_void_p(stream)
        self._fn = lib.leet_attn_forward_v3
        self.out = out

    def __call__(self) -> torch.Tensor:
        if torch.cuda.current_device() != self._dev.index:
            raise ValueError("PreparedForward called with another device current")
        stream = self._stream if self._stream is not None else ctypes.c_void_p(torch.cuda.current_stream(self._dev).cuda_stream)
        st = self._fn(*self._args, stream)
        if st != LEET_OK:
            raise LeetAttnError(st, "leet_attn_forward_v3")
        return self.out


def workspace_bytes_v3(B: int, H: int, N: int, r: int, dv: int, dtype: int, segments: int = 0,
                       kernel: int = LEET_CHOICE_DEFAULT) -> int:
    return int(lib.leet_attn_workspace_bytes_v3(B, H, N, r, dv, dtype, segments, kernel))


def query_plan_v3(B: int, H: int, N: int, r: int, dv: int, dtype: int, segments: int = 0,
                  kernel: int = LEET_CHOICE_DEFAULT):
    """``query_plan_rd`` with the kernel choice given per call."""
    nseg, kern = ctypes.c_int(0), ctypes.c_int(0)
    st = lib.leet_attn_query_plan_v3(B, H, N, r, dv, dtype, segments, kernel, ctypes.byref(nseg), ctypes.byref(kern))
    if st != LEET_OK:
        raise LeetAttnError(st, "leet_attn_query_plan_v3")
    return nseg.value, kern.value


def static_scratch_bytes() -> int:
    return int(lib.leet_attn_static_scratch_bytes())


def leet_attn_forward_static(q, k, v, gamma, out: torch.Tensor, state_in: Optional[torch.Tensor] = None,
                             state_out: Optional[torch.Tensor] = None, segments: int = 0) -> torch.Tensor:
    """Chunked prefill that allocates nothing: segment states in the library's static scratch.

    ``out`` is required (this binding allocates nothing for the call either)."""
    B, H, N, d = _check_forward(q, k, v, gamma, out)
    for name, s in (("state_in", state_in), ("state_out", state_out)):
        if s is not None and (s.dtype != torch.float32 or tuple(s.shape) != (B, H, d, d)):
            raise ValueError(f"{name} must be float32 [B, H, d, d]")
    dev = _check_dev(q, k, v, gamma, out, state_in, state_out)
    with torch.cuda.device(dev):
        st = lib.leet_attn_forward_static(_ptr(q), _ptr(k), _ptr(v), _ptr(gamma), _ptr(out), _ptr(state_in),
                                          _ptr(state_out), int(segments), B, H, N, d, _dtype_code(q),
                                          ctypes.c_void_p(_stream_ptr(dev)))
    if st != LEET_OK:
        raise LeetAttnError(st, "leet_attn_forward_static")
    return out


def leet_attn_forward_recurrent_rd(q, k, v, gamma: Optional[torch.Tensor], out: Optional[torch.Tensor] = None,
                                   state_in: Optional[torch.Tensor] = None,
                                   state_out: Optional[torch.Tensor] = None,
                                   mask: int = LEET_MASK_DECAY) -> torch.Tensor:
    """Row-based prefill with q, k of width r and v, out of width dv."""
    if out is None:
        out = torch.empty(v.shape, dtype=torch.float32, device=v.device)
    B, H, N, r, dv = _check_rd(q, k, v, gamma, out, False)
    _check_states_rd(B, H, r, dv, state_in=state_in, state_out=state_out)
    dev = _check_dev(q, k, v, gamma, out, state_in, state_out)
    with torch.cuda.device(dev):
        st = lib.leet_attn_forward_recurrent_rd(_ptr(q), _ptr(k), _ptr(v), _ptr(gamma), _ptr(out), _ptr(state_in),
                                                _ptr(state_out), B, H, N, r, dv, _dtype_code(q), int(mask),
                                                ctypes.c_void_p(_stream_ptr(dev)))
    if st != LEET_OK:
        raise LeetAttnError(st, "leet_attn_forward_recurrent_rd")
    return out


def leet_attn_forward_fleet(q, k, v, gamma: Optional[torch.Tensor], out: Optional[torch.Tensor] = None,
                            state_in: Optional[torch.Tensor] = None,
                            state_out: Optional[torch.Tensor] = None,
                            mask: int = LEET_MASK_DECAY) -> torch.Tensor:
    """FleetAttention prefill (rank-sum of discounted cumulative sums); q, k [B, H, N, r], v [B, H, N, dv]."""
    if out is None:
        out = torch.empty(v.shape, dtype=torch.float32, device=v.device)
    B, H, N, r, dv = _check_rd(q, k, v, gamma, out, False)
    _check_states_rd(B, H, r, dv, state_in=state_in, state_out=state_out)
    dev = _check_dev(q, k, v, gamma, out, state_in, state_out)
    with torch.cuda.device(dev):
        st = lib.leet_attn_forward_fleet(_ptr(q), _ptr(k), _ptr(v), _ptr(gamma), _ptr(out), _ptr(state_in),
                                         _ptr(state_out), B, H, N, r, dv, _dtype_code(q), int(mask),
                                         ctypes.c_void_p(_stream_ptr(dev)))
    if st != LEET_OK:
        raise LeetAttnError(st, "leet_attn_forward_fleet")
    return out


def leet_attn_decode_step_rd(q, k, v, gamma: Optional[torch.Tensor], state, out: Optional[torch.Tensor] = None,
                             mask: int = LEET_MASK_DECAY, store: Optional[int] = None) -> torch.Tensor:
    """One decode step with q, k [B, H, r], v [B, H, dv] and state [B, H, r, dv] (updated in place).

    ``store`` (a DECODE_STORE_* value) routes the call through ``leet_attn_decode_step_v3``, which takes
    the state store policy per call."""
    if q.dim() != 3 or q.shape != k.shape or v.dim() != 3 or q.shape[:2] != v.shape[:2]:
        raise ValueError("q, k must share one [B, H, r] shape and v be [B, H, dv]")
    if k.dtype != q.dtype or v.dtype != q.dtype:
        raise TypeError("q, k, v must share one dtype")
    B, H, r = q.shape
    dv = v.shape[2]
    if out is None:
        out = torch.empty(v.shape, dtype=torch.float32, device=v.device)
    if gamma is not None and (gamma.dtype != torch.float32 or gamma.numel() != H):
        raise ValueError("gamma must be float32 with one value per head")
    _check_states_rd(B, H, r, dv, state=state)
    if out.dtype != torch.float32 or tuple(out.shape) != (B, H, dv):
        raise ValueError("out must be float32 [B, H, dv]")
    dev = _check_dev(q, k, v, gamma, state, out)
    with torch.cuda.device(dev):
        if store is None:
            st = lib.leet_attn_decode_step_rd(_ptr(q), _ptr(k), _ptr(v), _ptr(gamma), _ptr(state), _ptr(out),
                                              B, H, r, dv, _dtype_code(q), int(mask), ctypes.c_void_p(_stream_ptr(dev)))
        else:
            st = lib.leet_attn_decode_step_v3(_ptr(q), _ptr(k), _ptr(v), _ptr(gamma), _ptr(state), _ptr(out),
                                              B, H, r, dv, _dtype_code(q), int(mask), int(store),
                                              ctypes.c_void_p(_stream_ptr(dev)))
    if st != LEET_OK:
        raise LeetAttnError(st, "leet_attn_decode_step_v3" if store is not None else "leet_attn_decode_step_rd")
    return out
