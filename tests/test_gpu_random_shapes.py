"""Seeded random shapes through every matmul path, checked on the device against a second route:
itq3s_dequantize (itself held to the oracle within 1e-6 elsewhere) followed by a dense fp64 product.
Cheap enough to visit hundreds of (M, N, K, dtype, zero-point pattern) combinations that the
oracle-based tests cannot afford; the bar is the same per-row relative L2."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

MS = [1, 2, 3, 4, 5, 7, 8, 9, 12, 16, 17, 20, 31, 32, 33, 48, 64, 100, 128, 129, 200, 256, 300, 512, 777]
KBS = [1, 2, 3, 4, 5, 8, 11, 16, 17, 20, 32, 33, 43, 56, 64, 80, 112, 144]
NS = [64, 100, 255, 256, 257, 500, 1000, 1024, 2047, 4096, 4100, 8192]


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_matmul_random_shapes_against_dequantize_and_dense_product(seed):
    import torch

    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_27914_amd import binding

    rng = np.random.default_rng(seed)
    g = torch.Generator(device="cuda")
    g.manual_seed(100 + seed)
    done = 0
    while done < 120:
        K, N, M = 256 * int(rng.choice(KBS)), int(rng.choice(NS)), int(rng.choice(MS))
        if N * K > 48e6 or M * K > 12e6:
            continue
        W = 0.02 * torch.randn((N, K), generator=g, device="cuda")
        if rng.random() < 0.5:  # rows with a constant offset in their first channel: zero-points in every block
            rows = torch.randint(0, N, (max(1, N // 50),), generator=g, device="cuda")
            W[rows, ::256] += 0.5 * torch.randn((rows.numel(), K // 256), generator=g, device="cuda")
        codes, scales = binding.itq3s_quantize(W)
        What = binding.itq3s_dequantize(codes, scales, N, K).double()
        X = torch.randn((M, K), generator=g, device="cuda").to(torch.float16)
        if rng.random() < 0.3:
            X[:, ::97] *= 10
        want = X.double() @ What.T
        for dtype, tol in ((torch.float32, 2e-3), (torch.float16, 2e-3)):
            got = binding.itq3s_matmul(codes, scales, N, K, X, dtype=dtype).double()
            assert bool(torch.isfinite(got).all()), (M, N, K, dtype)
            err = ((got - want).norm(dim=1) / want.norm(dim=1).clamp_min(1e-300)).max().item()
            assert err <= tol, (M, N, K, dtype, err)
        done += 1


@pytest.mark.parametrize("seed", [11, 12])
def test_other_matmul_routes_on_random_shapes(seed):
    """The same second route for the calls the test above does not reach: the weight-side kernel, the
    static-scratch entry point, and the sub-block-scale variant on all three of its paths (fused
    rotation, rotation launch, tiled weight-side kernel) against itq3s_dequantize_sub."""
    import torch

    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_27914_amd import binding

    rng = np.random.default_rng(seed)
    g = torch.Generator(device="cuda")
    g.manual_seed(200 + seed)

    def rel(got, want):
        return ((got.double() - want).norm(dim=1) / want.norm(dim=1).clamp_min(1e-300)).max().item()

    done = 0
    while done < 60:
        K, N, M = 256 * int(rng.choice(KBS)), int(rng.choice(NS)), int(rng.choice(MS))
        if N * K > 24e6 or M * K > 6e6:
            continue
        W = 0.02 * torch.randn((N, K), generator=g, device="cuda")
        W[:, :: int(rng.choice([37, 64, 256]))] *= float(rng.choice([1.0, 4.0, 12.0]))  # uneven sub-blocks after the rotation
        X = torch.randn((M, K), generator=g, device="cuda").to(torch.float16)
        dtype = torch.float16 if rng.random() < 0.5 else torch.float32
        codes, scales = binding.itq3s_quantize(W)
        want = X.double() @ binding.itq3s_dequantize(codes, scales, N, K).double().T
        assert rel(binding.itq3s_matmul_weight_side(codes, scales, N, K, X, dtype=dtype), want) <= 2e-3, ("weight side", M, N, K)
        if binding.itq3s_matmul_workspace_bytes(M, N, K) <= (64 << 20):  # the static array's size
            out = torch.empty((M, N), dtype=dtype, device="cuda")
            assert rel(binding.itq3s_matmul_static(codes, scales, N, K, X, out), want) <= 2e-3, ("static", M, N, K)
        c2, s2, u2 = binding.itq3s_quantize_sub(W)
        want2 = X.double() @ binding.itq3s_dequantize_sub(c2, s2, u2, N, K).double().T
        assert rel(binding.itq3s_matmul_sub(c2, s2, u2, N, K, X, dtype=dtype), want2) <= 2e-3, ("sub", M, N, K)
        done += 1
