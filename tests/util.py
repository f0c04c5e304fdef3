"""Helpers shared by the GPU parity tests (uploads, comparisons); no method arithmetic."""
import numpy as np
import torch

from oracle import ecospa_oracle as O
from paper_2511_11641_amd import binding as B

TOL = {"f32": 1e-5, "bf16": 2e-2}     # relative Frobenius error bounds of the two storage types
TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16}


def dev(a, dtype="f32"):
    """numpy float32 (already rounded to the storage dtype) -> cuda tensor of that dtype."""
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a))
    if t.dtype == torch.float32:
        t = t.to(TORCH_DT[dtype])
    return t.cuda()


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


ROW_FACTOR = 8.0      # a single row or column may be this many times worse than the whole tensor's bound
ELEM_FACTOR = 16.0    # ... and a single element this many, relative to the tensor's RMS element


def assert_close(got, want, dtype, what=""):
    """The stated tolerance is the relative Frobenius error of the whole tensor.  A norm over everything would let
    one bad row, one bad column (a tile edge) or one garbage element of a large output through, so three local bounds
    stand beside it: every row's and every column's error against the RMS row / column norm of the expected tensor
    (ROW_FACTOR x tolerance), and every element's error against the RMS element (ELEM_FACTOR x tolerance)."""
    g = host(got) if isinstance(got, torch.Tensor) else np.asarray(got, dtype=np.float64)
    w = np.asarray(want, dtype=np.float64)
    assert g.shape == w.shape, f"{what}: shape {g.shape} != {w.shape}"
    tol = TOL[dtype]
    err = O.rel_fro(g, w)
    assert err <= tol, f"{what}: rel Frobenius error {err:.3e} > {tol:.0e}"
    fro = float(np.sqrt((w * w).sum()))
    if fro > 0.0 and w.size > 1:
        diff = g - w
        rms = fro / np.sqrt(w.size)
        worst = float(np.abs(diff).max())
        assert worst <= ELEM_FACTOR * tol * rms, \
            f"{what}: element error {worst:.3e} > {ELEM_FACTOR * tol:.1e} x RMS element {rms:.3e} at {np.unravel_index(np.abs(diff).argmax(), w.shape)}"
        if w.ndim >= 2:
            d2 = diff.reshape(-1, w.shape[-1])
            rows, cols = d2.shape
            row_err = np.sqrt((d2 * d2).sum(axis=1)) / (fro / np.sqrt(rows))
            col_err = np.sqrt((d2 * d2).sum(axis=0)) / (fro / np.sqrt(cols))
            assert row_err.max() <= ROW_FACTOR * tol, \
                f"{what}: row {int(row_err.argmax())} error {row_err.max():.3e} > {ROW_FACTOR * tol:.1e} (of the RMS row norm)"
            assert col_err.max() <= ROW_FACTOR * tol, \
                f"{what}: column {int(col_err.argmax())} error {col_err.max():.3e} > {ROW_FACTOR * tol:.1e} (of the RMS column norm)"
    return err


def pad_rows(a, groups, k, kp):
    """Oracle compact rows [groups*k, c] -> padded layout [groups*kp, c] with zero rows."""
    a = np.asarray(a)
    out = np.zeros((groups * kp,) + a.shape[1:], dtype=a.dtype)
    out.reshape(groups, kp, *a.shape[1:])[:, :k] = a.reshape(groups, k, *a.shape[1:])
    return out


def pad_cols(a, groups, k, kp):
    return np.ascontiguousarray(pad_rows(np.asarray(a).T, groups, k, kp).T)


def interleave_rows(a, b):
    """Rows a[0], b[0], a[1], b[1], ...: the compact layout of a gated FFN's first matrix (gate unit i in row 2i, up
    unit i in row 2i + 1) from its two halves."""
    a, b = np.asarray(a), np.asarray(b)
    out = np.empty((2 * a.shape[0],) + a.shape[1:], dtype=a.dtype)
    out[0::2], out[1::2] = a, b
    return out
