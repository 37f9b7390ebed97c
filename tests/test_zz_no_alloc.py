"""itq3s_matmul_static (scratch in the library's static device array, nothing allocated) against
itq3s_matmul with a caller-provided workspace: same kernels, so the outputs are bit-identical.  Two
calls in a row on the shared array, the second with a smaller input; paths that use the scratch
(5..16 rows: rotated activations; more rows: rotated activations, split-K shares and their flags)
and the one that does not (M <= 4)."""
import ctypes

import numpy as np
import pytest

from paper_2603_27914_amd import synth
from tests.packed_inputs import random_packed

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch

    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_27914_amd import binding

    binding.lib()
    return torch, binding


def dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def static_call(torch, binding, cd, sd, N, K, X, out):
    """Straight through the C ABI (device pointers and sizes only)."""
    L = binding.lib()
    rc = L.itq3s_matmul_static(ctypes.c_void_p(cd.data_ptr()), ctypes.c_void_p(sd.data_ptr()), N, K, ctypes.c_void_p(X.data_ptr()), X.shape[0], X.stride(0),
                               ctypes.c_void_p(out.data_ptr()), binding.F16 if out.dtype == torch.float16 else binding.F32, out.stride(0), None,
                               ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    return rc


@pytest.mark.parametrize("first,second", [((300, 600, 2048), (40, 200, 1024)),   # tiled path with split-K shares, twice
                                          ((16, 1000, 4096), (7, 333, 1024)),    # rotation launch + streaming kernel
                                          ((512, 4096, 4096), (3, 96, 512)),     # large tiled call, then the path without scratch
                                          ((64, 272, 11008), (9, 48, 768))])
def test_static_scratch_matches_workspace_variant(gpu, ref, first, second):
    torch, binding = gpu
    for i, (M, N, K) in enumerate((first, second)):
        codes, scales = random_packed(N, K, "static", M, z_fraction=0.02)
        cd, sd = dev(torch, codes.view(np.int32)), dev(torch, scales.view(np.int32))
        X = synth.activations(M, K, "static", M)
        Xd = dev(torch, X)
        for dtype in (torch.float32, torch.float16):
            want = binding.itq3s_matmul(cd, sd, N, K, Xd, dtype=dtype)
            got = torch.full((M, N), float("nan"), dtype=dtype, device="cuda")
            assert static_call(torch, binding, cd, sd, N, K, Xd, got) == 0
            torch.cuda.synchronize()
            assert torch.equal(got, want), (i, M, N, K, dtype)
        # and against the oracle on a few output columns, to the bar of every other matmul test
        n1 = min(N, 24)
        Yr = ref.matmul(codes, scales, N, K, X, rows=(0, n1))[:, :n1]
        Y = got.float().cpu().numpy()[:, :n1].astype(np.float64)
        err = np.max(np.linalg.norm(Y - Yr, axis=1) / np.linalg.norm(Yr, axis=1))
        assert err <= 2e-3, err


def test_static_scratch_rejects_what_does_not_fit(gpu):
    torch, binding = gpu
    L = binding.lib()
    M, N, K = 4096, 64, 16384  # 128 MiB of rotated activations
    assert L.itq3s_matmul_workspace_bytes(M, N, K) > (64 << 20)
    codes, scales = random_packed(N, K, "static-big")
    cd, sd = dev(torch, codes.view(np.int32)), dev(torch, scales.view(np.int32))
    X = torch.zeros((M, K), dtype=torch.float16, device="cuda")
    out = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    assert static_call(torch, binding, cd, sd, N, K, X, out) == -5
    with pytest.raises(binding.Itq3sError, match="workspace"):
        binding.itq3s_matmul_static(cd, sd, N, K, X, out)
