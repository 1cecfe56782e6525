"""The entry point that allocates nothing (clover_op_gemm_static: scratch in a fixed device array inside the
library) against the entry point it is a variant of (clover_op_gemm with caller-provided scratch)."""
import ctypes as C

import numpy as np
import pytest

from paper_2408_00264_amd import clover, synth

pytestmark = pytest.mark.gpu


def _run(lib, torch, static, path, M, N, K, seed):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((M, K)).astype(np.float32)
    Wb = synth.f32_to_bf16_bits((rng.standard_normal((N, K)) * 0.02).astype(np.float32))
    Xd = torch.from_numpy(X).cuda()
    Wd = torch.from_numpy(Wb.view(np.int16)).cuda()
    Y = torch.full((M, N), -3.0, dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    if static:
        rc = lib.clover_op_gemm_static(path, 1, C.c_void_p(Xd.data_ptr()), C.c_void_p(Wd.data_ptr()),
                                       C.c_void_p(Y.data_ptr()), N, M, N, K, C.c_void_p(st))
    else:
        nb = lib.clover_op_gemm_scratch_bytes(M, N, K)
        scratch = torch.zeros(nb, dtype=torch.uint8, device="cuda")
        rc = lib.clover_op_gemm(path, 1, C.c_void_p(Xd.data_ptr()), C.c_void_p(Wd.data_ptr()),
                                C.c_void_p(Y.data_ptr()), N, M, N, K, C.c_void_p(scratch.data_ptr()), nb, C.c_void_p(st))
    assert rc == 0, lib.clover_last_global_error()
    torch.cuda.synchronize()
    ref = X.astype(np.float64) @ synth.bf16_bits_to_f32(Wb).astype(np.float64).T
    return Y.cpu().numpy(), ref


@pytest.mark.parametrize("path", [1, 3], ids=["k_slice", "panel"])
def test_static_scratch_gemm_matches_caller_scratch_gemm(path):
    import torch
    assert torch.cuda.is_available()
    lib = clover.load_library()
    # two calls in a row on the shared array, the second with a smaller input: stale contents of the first
    # (weight copy, activation planes, partial sums) must not leak into the second
    shapes = [(64, 2048, 2048), (37, 512, 1024)]
    for i, (M, N, K) in enumerate(shapes):
        print(f"static-scratch gemm path {path}: M={M} N={N} K={K}", flush=True)
        assert lib.clover_op_gemm_scratch_bytes(M, N, K) <= clover.STATIC_SCRATCH_BYTES
        got, ref = _run(lib, torch, True, path, M, N, K, seed=100 + i)
        want, _ = _run(lib, torch, False, path, M, N, K, seed=100 + i)
        np.testing.assert_array_equal(got, want)                    # same kernels, same inputs: same bits
        tol = 4e-5 * np.sqrt(K) * 0.02 * 4                          # and both within the MFMA path's bound
        assert np.abs(got - ref).max() <= tol


def test_static_scratch_limits():
    import torch
    assert torch.cuda.is_available()
    lib = clover.load_library()
    x = torch.zeros(16, dtype=torch.float32, device="cuda")
    p = C.c_void_p(x.data_ptr())
    # too large for the array: refused on the host, nothing launched
    assert lib.clover_op_gemm_scratch_bytes(64, 8192, 8192) > clover.STATIC_SCRATCH_BYTES
    assert lib.clover_op_gemm_static(1, 1, p, p, p, 8192, 64, 8192, 8192, None) == clover.E_CAPACITY
    assert b"CLOVER_STATIC_SCRATCH_BYTES" in lib.clover_last_global_error()
    # the copy-reusing paths make no sense on a shared array
    assert lib.clover_op_gemm_static(2, 1, p, p, p, 512, 16, 512, 512, None) == clover.E_SHAPE
