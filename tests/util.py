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


def assert_close(got, want, dtype, what=""):
    err = O.rel_fro(host(got) if isinstance(got, torch.Tensor) else got, want)
    assert err <= TOL[dtype], f"{what}: rel Frobenius error {err:.3e} > {TOL[dtype]:.0e}"
    return err


def pad_rows(a, groups, k, kp):
    """Oracle compact rows [groups*k, c] -> padded layout [groups*kp, c] with zero rows."""
    a = np.asarray(a)
    out = np.zeros((groups * kp,) + a.shape[1:], dtype=a.dtype)
    out.reshape(groups, kp, *a.shape[1:])[:, :k] = a.reshape(groups, k, *a.shape[1:])
    return out


def pad_cols(a, groups, k, kp):
    return np.ascontiguousarray(pad_rows(np.asarray(a).T, groups, k, kp).T)
