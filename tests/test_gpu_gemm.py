"""GPU parity of the layer's bf16 MFMA GEMM (Method, Eq. 1: every linear map of the frozen layer) against the plain
definition: c[m][n] = sum_k a[m][k] * w[n][k] in fp64 on the bf16-rounded operands. The shapes walk the corners of
the kernel's pipeline: the shortest K (two slices), K of an odd number of slice pairs, a ragged last row tile, one
tile, and grids with more tiles than compute units (one persistent workgroup per CU walks several tiles, with and
without a remainder)."""
import numpy as np
import pytest
import torch

from paper_2605_10875_amd import sol, synth

from gpu_util import host

pytestmark = pytest.mark.gpu


def _bf16(x):
    return synth.round_to_bf16(x.astype(np.float32))


@pytest.mark.parametrize("M,N,K", [(256, 256, 128), (256, 256, 256), (300, 512, 384), (1, 256, 128), (77, 768, 640),
                                   (8192, 2560, 128), (8192, 2560, 384), (8448, 2048, 256), (8200, 2560, 256)])
def test_gemm_matches_the_definition(M, N, K):
    rng = np.random.default_rng(M * 31 + N * 7 + K)
    a = _bf16(rng.standard_normal((M, K)))
    w = _bf16(rng.standard_normal((N, K)) * 0.1)
    c = host(sol.gemm(torch.from_numpy(a).cuda().to(torch.bfloat16), torch.from_numpy(w).cuda().to(torch.bfloat16)))
    ref = a.astype(np.float64) @ w.astype(np.float64).T
    # fp32 accumulation of K products of magnitude |a||w|: error far below 1e-5 of the row scale
    scale = np.abs(a).astype(np.float64) @ np.abs(w).astype(np.float64).T
    err = np.abs(c - ref) / np.maximum(scale, 1e-30)
    assert np.isfinite(c).all() and err.max() < 1e-5, (err.max(), np.unravel_index(err.argmax(), err.shape))


def test_gemm_rejects_shapes_outside_the_kernel():
    a = torch.zeros((64, 192), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((256, 192), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sol.SolError):
        sol.gemm(a, w)                      # K not a multiple of 128
    a = torch.zeros((64, 128), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((192, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sol.SolError):
        sol.gemm(a, w)                      # N not a multiple of 256
