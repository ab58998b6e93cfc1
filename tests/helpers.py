"""Shared test helpers: error metrics and golden-file parsing (no operator arithmetic)."""
import numpy as np


def rel_err_per_head(got, ref):
    """max|got-ref| / max|ref| per (b,h) slab; arrays are [B,H,...]. Returns [B,H]."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    B, H = ref.shape[:2]
    g = got.reshape(B, H, -1)
    r = ref.reshape(B, H, -1)
    num = np.abs(g - r).max(axis=2)
    den = np.abs(r).max(axis=2)
    den = np.where(den > 0, den, 1.0)
    return num / den


def max_rel_err(got, ref):
    """Worst (b,h) of ``rel_err_per_head``: the primary parity metric."""
    return float(rel_err_per_head(got, ref).max())


def elementwise_ok(got, ref, tol):
    """Secondary metric: |got-ref| <= tol * (|ref| + rms(ref)) element by element, rms per (b,h)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    B, H = ref.shape[:2]
    g = got.reshape(B, H, -1)
    r = ref.reshape(B, H, -1)
    rms = np.sqrt((r * r).mean(axis=2, keepdims=True))
    return bool(np.all(np.abs(g - r) <= tol * (np.abs(r) + rms) + 1e-300))


def elementwise_ok_windowed(got, ref, tol, window=64):
    """The element-wise bound with the rms taken over the window of `window` tokens that the element
    sits in (per (b,h)), for [B,H,N,d] arrays: |got-ref| <= tol * (|ref| + rms_window(ref)).

    The rounding errors of the 16-bit kernels scale with the operands of the moment -- the state is
    rounded to the input type once per 64-token chunk -- so where the output scale changes along the
    sequence (a large entering state on a fast-decaying head) the scale that an error must be held
    against is the local one, not the rms of the whole head.  Tighter than the per-head bound where
    the outputs are small, looser where they are large."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    B, H, N, d = ref.shape
    ok = True
    for t0 in range(0, N, window):
        r = ref[:, :, t0:t0 + window].reshape(B, H, -1)
        g = got[:, :, t0:t0 + window].reshape(B, H, -1)
        rms = np.sqrt((r * r).mean(axis=2, keepdims=True))
        ok = ok and bool(np.all(np.abs(g - r) <= tol * (np.abs(r) + rms) + 1e-300))
    return ok


def parse_golden(path):
    """'name a b ; c d' lines -> dict name -> 2-D float array (1-D rows for single-row entries)."""
    out = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, rest = line.split(None, 1)
            rows = [[float(x) for x in row.split()] for row in rest.split(";")]
            out[name] = np.array(rows, dtype=np.float64)
    return out
