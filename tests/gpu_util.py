"""Helpers shared by the GPU parity tests: host arrays <-> device tensors, error metrics."""
import numpy as np
import torch

from paper_2605_10875_amd import sol


def tdtype(dtype_code):
    return torch.bfloat16 if dtype_code == sol.BF16 else torch.float32


def dev(a, dtype_code=None):
    """numpy -> cuda tensor. float arrays go to the storage dtype (values are expected to be
    representable there already), integer arrays to int32."""
    if np.issubdtype(a.dtype, np.integer):
        return torch.from_numpy(np.ascontiguousarray(a, np.int32)).cuda()
    t = torch.from_numpy(np.ascontiguousarray(a, np.float32)).cuda()
    return t.to(tdtype(dtype_code)).contiguous() if dtype_code is not None else t


def dev_weights(w, dtype_code):
    return {k: dev(v, dtype_code) for k, v in w.items()}


def host(t):
    return t.detach().float().cpu().numpy()


def rel_err(got, ref):
    """max |got - ref| / max |ref| over the tensor (element-wise relative error is meaningless near 0)."""
    ref = np.asarray(ref, np.float64)
    got = np.asarray(got, np.float64)
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def frac_mismatch(got, ref, tol):
    ref = np.asarray(ref, np.float64)
    got = np.asarray(got, np.float64)
    return float((np.abs(got - ref) > tol * np.abs(ref).max()).mean())


def check_rows(got, ref, tight, loose, max_bad_frac, what="", median=None):
    """Row-wise comparison that tolerates the method's discontinuities: a quantisation code or a
    selected key / channel that flips at a rounding boundary moves one token row by a bounded
    amount. Every row must be within `loose` (max-rel against the tensor's max |ref|); at most
    `max_bad_frac` of the rows may exceed `tight`."""
    ref = np.asarray(ref, np.float64)
    got = np.asarray(got, np.float64)
    scale = max(np.abs(ref).max(), 1e-30)
    err = np.abs(got - ref).reshape(-1, ref.shape[-1]).max(axis=1) / scale
    worst = float(err.max())
    bad = float((err > tight).mean())
    med = float(np.median(err))
    msg = (f"{what}: median row {med:.2e}, worst row {worst:.3e} (cap {loose:.1e}); "
           f"rows over {tight:.1e}: {bad:.4f} (allowed {max_bad_frac})")
    print(msg)
    assert worst < loose, msg
    assert bad <= max_bad_frac, msg
    if median is not None:
        assert med < median, msg
