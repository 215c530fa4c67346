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


def check_by_bit_class(out, ref_bf16, ref_fp32, ids, table, what, full_size=False, pages=False):
    """Layer outputs by the bit-width class of the row's action, against both storage modes of the oracle.

    Rows of quantising actions cross four quantisers and three contractions inside the layer; a code that flips at a
    rounding boundary is a jump of 1 / q_max of the row's range and the next contraction spreads it, so two correct
    implementations that differ in summation order disagree on such rows by percents (the stage-wise tests, which
    feed each stage the oracle's inputs, are where these rows are bounded tightly). The yardstick here is the oracle
    itself: its bf16-store and fp32-store modes are two correct evaluations of the same layer that differ by one
    bf16 rounding per hand-over, a perturbation of the same kind as, and larger than, the GPU's fp32-versus-fp64
    sums. Per class the GPU must be no further from the bf16-store oracle than the fp32-store oracle is (median and
    90th percentile of the row errors, with a quarter of slack), every row stays under the cap of six quantisation
    steps, and rows of non-quantising actions are held to the contract itself: every row within 2e-2 of the
    bf16-store oracle (full-size runs: 1 % of rows up to 5e-2, 5 % under the page rule, one swapped key or page of a
    short row), median within 1e-2; against the fp32-store oracle the same rows: median within 1e-2 and no more rows
    over 2e-2 than the two oracles have between them (half as many again, plus 1 %)."""
    ref_bf16, out = np.asarray(ref_bf16, np.float64), np.asarray(out, np.float64)
    scale = max(np.abs(ref_bf16).max(), 1e-30)
    bits = np.array([a[4] for a in table])[ids]
    e_gpu = np.abs(out - ref_bf16).max(axis=-1) / scale
    if ref_fp32 is None:             # no fp32-store leg (the largest full-size cases): the cap and the contract only
        for b in sorted(set(bits.reshape(-1).tolist())):
            g = e_gpu[bits == b]
            msg = (f"{what}: rows of {b}-bit actions ({g.size}): gpu vs bf16-store oracle median {np.median(g):.2e} "
                   f"q90 {np.quantile(g, .9):.2e} max {g.max():.2e} over 2e-2: {(g > 2e-2).mean():.3f}")
            print(msg)
            if b >= 16:
                assert np.median(g) < 1e-2 and g.max() < 5e-2 and (g > 2e-2).mean() <= (0.05 if pages else 0.01), msg
            else:
                assert g.max() < max(2e-2, 6.0 / 2 ** (b - 1)), msg
        return
    ref_fp32 = np.asarray(ref_fp32, np.float64)
    e_gpu32 = np.abs(out - ref_fp32).max(axis=-1) / scale
    e_orc = np.abs(ref_bf16 - ref_fp32).max(axis=-1) / scale
    for b in sorted(set(bits.reshape(-1).tolist())):
        g, g32, o = e_gpu[bits == b], e_gpu32[bits == b], e_orc[bits == b]
        msg = (f"{what}: rows of {b}-bit actions ({g.size}): gpu vs bf16-store oracle median {np.median(g):.2e} "
               f"q90 {np.quantile(g, .9):.2e} max {g.max():.2e} over 2e-2: {(g > 2e-2).mean():.3f} | fp32-store vs bf16-store "
               f"oracle median {np.median(o):.2e} q90 {np.quantile(o, .9):.2e} max {o.max():.2e} | gpu vs fp32-store oracle "
               f"median {np.median(g32):.2e} over 2e-2: {(g32 > 2e-2).mean():.3f} (oracles: {(o > 2e-2).mean():.3f})")
        print(msg)
        if b >= 16:
            assert np.median(g) < 1e-2, msg
            if full_size:
                assert g.max() < 5e-2 and (g > 2e-2).mean() <= (0.05 if pages else 0.01), msg
            else:
                assert g.max() < 2e-2, msg
            assert np.median(g32) < 1e-2 and (g32 > 2e-2).mean() <= 1.5 * (o > 2e-2).mean() + 0.01, msg
            assert g32.max() <= 1.5 * max(o.max(), 2e-2), msg
        else:
            cap = max(2e-2, 6.0 / 2 ** (b - 1))
            assert g.max() < cap, msg
            assert np.median(g) <= 1.25 * np.median(o) + 1e-3, msg
            assert np.quantile(g, .9) <= 1.25 * np.quantile(o, .9) + 1e-3, msg
