"""HIP path vs CPU oracle, through the C ABI (ctypes binding).  Needs a real MI355X: -m gpu.

Bars: packed codes and scale words bit-exact; dequantize <= 1e-6 relative L2 per row (fp32 out);
matmul <= 2e-3 relative L2 per activation row against the oracle's fp64 result computed from the
same packed bytes."""
import numpy as np
import pytest

from paper_2603_27914_amd import synth
from tests.packed_inputs import random_packed, unpack_numpy

pytestmark = pytest.mark.gpu

MATMUL_TOL = 2e-3
DEQ_TOL = 1e-6


@pytest.fixture(scope="module")
def gpu():
    import torch

    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_27914_amd import binding

    binding.lib()  # fails loudly if the HIP library is not built
    return torch, binding


def to_dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def u32(t):
    return t.cpu().numpy().view(np.uint32)


def rel_rows(got, want):
    num = np.linalg.norm(got.astype(np.float64) - want, axis=1)
    den = np.linalg.norm(want, axis=1)
    return np.max(num / np.maximum(den, 1e-300))


# ----------------------------------------------------------------------------------- quantize


def check_quantize(torch, binding, ref, W, ldw=None):
    N, K = W.shape
    if ldw is None:
        Wd = to_dev(torch, W)
    else:
        buf = torch.zeros((N, ldw), dtype=torch.float32, device="cuda")
        buf[:, :K] = to_dev(torch, W)
        Wd = buf[:, :K]
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    codes, scales = binding.itq3s_quantize(Wd, status_flags=flags)
    torch.cuda.synchronize()
    rc, rs, rflags = ref.quantize(W)
    assert np.array_equal(u32(scales), rs), "scale words differ"
    assert np.array_equal(u32(codes), rc), "packed codes differ"
    assert int(flags.item()) == rflags
    return codes, scales


def test_quantize_config1_bit_exact(gpu, ref):
    torch, binding = gpu
    W = synth.weights(2048, 2048, "single", n_outlier_cols=4)
    check_quantize(torch, binding, ref, W)


@pytest.mark.parametrize("N,K,ldw", [(1, 256, None), (40, 768, None), (17, 512, 520), (333, 1024, None)])
def test_quantize_ragged_shapes(gpu, ref, N, K, ldw):
    torch, binding = gpu
    check_quantize(torch, binding, ref, synth.weights(N, K, "ragged", n_outlier_cols=2), ldw)


def test_quantize_adversarial_blocks(gpu, ref):
    torch, binding = gpu
    rng = np.random.default_rng(42)
    rows = []
    rows.append(np.zeros(256, np.float32))  # all zero
    rows.append(np.full(256, 0.37, np.float32))  # constant
    e0 = np.zeros(256, np.float32); e0[0] = 3.0; rows.append(e0)  # spike at 0: sigma = 0
    e5 = np.zeros(256, np.float32); e5[5] = -7.0; rows.append(e5)  # spike elsewhere
    rows.append((rng.standard_normal(256) * 1e6).astype(np.float32))  # scale saturates
    rows.append((rng.standard_normal(256) * 1e-7).astype(np.float32))  # subnormal fp16 scale
    rows.append((rng.standard_normal(256) * 1e-9).astype(np.float32))  # scale underflows to 0
    w = (rng.standard_normal(256) * 1e-3).astype(np.float32); w[0] = 1e3; rows.append(w)  # z clamps
    w = (0.02 * rng.standard_t(4, 256)).astype(np.float32); w[0] = 0.9; rows.append(w)  # z != 0
    w = (0.02 * rng.standard_t(4, 256)).astype(np.float32); w[0] = -1.7; rows.append(w)  # z != 0, other sign
    w = rng.standard_normal(256).astype(np.float32); w[17] = np.inf; rows.append(w)
    w = rng.standard_normal(256).astype(np.float32); w[200] = np.nan; rows.append(w)
    rows.append(np.full(256, np.finfo(np.float32).max, np.float32) * np.sign(rng.standard_normal(256)).astype(np.float32))
    rows.append((rng.standard_normal(256) * np.finfo(np.float32).tiny).astype(np.float32))  # fp32 subnormal range
    # integer-valued transform-domain data: coefficients land exactly on decision thresholds
    for _ in range(20):
        target = rng.integers(-40, 41, size=256).astype(np.float64) * 16.0
        rows.append((ref.fwht256(target) / 256.0).astype(np.float32))
    W = np.stack(rows)
    for K in (256,):
        check_quantize(torch, binding, ref, W)
    # the same blocks side by side in one row-major matrix with three block columns
    W3 = np.concatenate([W, W[::-1], np.roll(W, 3, axis=0)], axis=1)
    check_quantize(torch, binding, ref, W3)


def test_quantize_blocks_across_the_whole_fp32_range(gpu, ref):
    """Blocks at every magnitude an fp32 can hold (subnormal to the largest finite numbers), and blocks
    whose elements span ten decades: the kernel applies the transform's power-of-two factor to the
    block's scalars instead of its elements, which is bit-identical only as long as no intermediate
    value leaves the fp64 range -- checked here against the oracle, which scales the elements."""
    torch, binding = gpu
    rng = np.random.default_rng(7)
    rows = []
    with np.errstate(over="ignore", under="ignore"):
        for e in range(-45, 39):
            for _ in range(24):
                rows.append((rng.standard_normal(256) * 10.0**e).astype(np.float32))
            for _ in range(8):
                rows.append((rng.standard_normal(256) * 10.0 ** (e + rng.uniform(-5, 5, size=256))).astype(np.float32))
    W = np.nan_to_num(np.stack(rows), nan=0.0, posinf=np.finfo(np.float32).max, neginf=-np.finfo(np.float32).max)
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    codes, scales = binding.itq3s_quantize(to_dev(torch, W), status_flags=flags)
    torch.cuda.synchronize()
    rc, rs, rflags = ref.quantize(W)
    assert np.array_equal(u32(scales), rs), "scale words differ"
    assert np.array_equal(u32(codes), rc), "packed codes differ"
    assert int(flags.item()) == rflags


def test_quantize_many_random_blocks(gpu, ref):
    """Half a million heavy-tailed blocks: any disagreement in rounding (sqrt, division, the two
    conversion steps of the scale, the summation order) would flip a scale bit or a code somewhere."""
    torch, binding = gpu
    W = synth.weights(4096, 4096 * 8, "many", n_outlier_cols=33)
    check_quantize(torch, binding, ref, W)


# ----------------------------------------------------------------------------------- dequantize


@pytest.mark.parametrize("N,K", [(16, 256), (40, 768), (2048, 2048)])
def test_dequantize_fp32(gpu, ref, N, K):
    torch, binding = gpu
    W = synth.weights(N, K, "deq", n_outlier_cols=4)
    W[:, 0] += 0.5  # non-zero zero-points in the first block column
    codes, scales, _ = ref.quantize(W)
    want = ref.dequantize(codes, scales, N, K)
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    got = binding.itq3s_dequantize(to_dev(torch, codes.view(np.int32)), to_dev(torch, scales.view(np.int32)), N, K, status_flags=flags)
    got = got.cpu().numpy()
    assert int(flags.item()) == 0
    assert rel_rows(got, want) <= DEQ_TOL
    # element-wise: one fp32 rounding of an exactly known product
    assert np.max(np.abs(got - want) / np.maximum(np.abs(want), 1e-30)) <= 2.0**-23


def test_dequantize_fp16_and_strided(gpu, ref):
    torch, binding = gpu
    N, K = 100, 512
    codes, scales = random_packed(N, K, "deq16", z_fraction=0.05)
    want = ref.dequantize(codes, scales, N, K)
    cd, sd = to_dev(torch, codes.view(np.int32)), to_dev(torch, scales.view(np.int32))
    buf = torch.zeros((N, K + 8), dtype=torch.float16, device="cuda")
    binding.itq3s_dequantize(cd, sd, N, K, out=buf[:, :K])
    got = buf.cpu().numpy()
    assert not got[:, K:].any()
    # fp16 output: within one fp16 rounding of the exact value (the kernel rounds through fp32)
    w16 = want.astype(np.float16).astype(np.float64)
    ulp = np.maximum(np.abs(np.spacing(want.astype(np.float16)).astype(np.float64)), 2.0**-24)
    assert np.all(np.abs(got[:, :K].astype(np.float64) - w16) <= ulp)
    assert rel_rows(got[:, :K], want) <= 1e-3


def test_dequantize_flags_bad_codes(gpu, ref):
    torch, binding = gpu
    codes, scales = random_packed(32, 512, "bad")
    for word, bit in ((7, 3 << 10), (256 + 40, 1 << 9)):
        bad = codes.copy()
        bad[384 * 2 + word] |= np.uint32(bit)
        flags = torch.zeros(1, dtype=torch.int32, device="cuda")
        got = binding.itq3s_dequantize(to_dev(torch, bad.view(np.int32)), to_dev(torch, scales.view(np.int32)), 32, 512, status_flags=flags)
        want, rflags = ref.dequantize(bad, scales, 32, 512, return_flags=True)
        assert int(flags.item()) == rflags == binding.FLAG_BAD_CODE
        assert rel_rows(got.cpu().numpy(), want) <= DEQ_TOL


def test_quantize_dequantize_round_trip_error_bound(gpu, ref):
    """Thm 2 on the GPU path: per block, ||w_hat - w||^2 <= sum_j max(d/2, |w'_j/d + z| - 1)^2 d^2."""
    torch, binding = gpu
    N, K = 64, 1024
    W = synth.weights(N, K, "rt")
    codes, scales = binding.itq3s_quantize(to_dev(torch, W))
    What = binding.itq3s_dequantize(codes, scales, N, K).cpu().numpy().astype(np.float64)
    s = u32(scales).reshape(-1, 4, 16)
    for n in range(0, N, 7):
        for b in range(4):
            word = int(s[n // 16, b, n % 16])
            d = float(np.array([word & 0xFFFF], np.uint16).view(np.float16)[0])
            z = float(np.array([word >> 16], np.uint16).view(np.float16)[0])
            wt = ref.forward_block(W[n, 256 * b : 256 * b + 256])
            bound = np.sum((np.maximum(0.5, np.abs(wt / d + z) - 1.0) * d) ** 2)
            err = np.sum((What[n, 256 * b : 256 * b + 256] - W[n, 256 * b : 256 * b + 256]) ** 2)
            assert err <= bound * (1 + 1e-5)


# ----------------------------------------------------------------------------------- matmul


def run_matmul(torch, binding, ref, codes, scales, N, K, X, out_dtype=None, rows=None):
    cd, sd = to_dev(torch, codes.view(np.int32)), to_dev(torch, scales.view(np.int32))
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    Y = binding.itq3s_matmul(cd, sd, N, K, to_dev(torch, X), dtype=out_dtype or torch.float32, status_flags=flags)
    torch.cuda.synchronize()
    assert int(flags.item()) == 0
    out_f16 = Y.dtype == torch.float16
    Y = Y.float().cpu().numpy()
    if rows is None:
        want = ref.matmul(codes, scales, N, K, X)
        check_elements(Y, want, codes, scales, N, K, X, out_f16)
        return rel_rows(Y, want)
    worst = 0.0
    for n0, n1 in rows:
        want = ref.matmul(codes, scales, N, K, X, rows=(n0, n1))[:, n0:n1]
        worst = max(worst, rel_rows(Y[:, n0:n1], want))
    return worst


def check_elements(Y, want, codes, scales, N, K, X, out_f16=False):
    """Bound on every single element, next to the per-row bar: the kernels round the rotated
    activations once to fp16 (relative 2^-11 each) and multiply them with the exact digits d q, the
    zero-point term is formed in fp32 from the activations themselves, so
        |Y[m,n] - want[m,n]| <= 2^-11 sum_k |d q[n,k]| |x~[m,k]| <= 2^-11 ||d q[n,:]|| ||x[m,:]||
    (Cauchy-Schwarz; ||x~|| = ||x||, the rotation is orthogonal), plus the fp32 accumulation and the
    rounding of the output.  A single wrong digit or scale in a short row breaks it."""
    c, d, z = unpack_numpy(np.asarray(codes), np.asarray(scales), N, K)
    dq = (c - 1).astype(np.float64) * np.repeat(d, 256, axis=1)
    wn = np.linalg.norm(dq, axis=1)                      # [N]
    xn = np.linalg.norm(X.astype(np.float64), axis=1)    # [M]
    bound = 1.5 * 2.0 ** -11 * xn[:, None] * wn[None, :] + 2.0 ** (-11 if out_f16 else -22) * np.abs(want) + 1e-30
    err = np.abs(Y.astype(np.float64) - want)
    worst = np.max(err / bound)
    assert worst <= 1.0, "an element misses its bound by a factor %.2f" % worst


@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 8, 11, 16, 17, 25, 32])  # 17..32: two passes of the streaming kernel
@pytest.mark.parametrize("N,K", [(16, 256), (48, 512), (1000, 1024), (2048, 2048), (1160, 4096), (272, 11008), (100, 20480), (40, 36864)])
def test_matmul_small_m(gpu, ref, M, N, K):
    torch, binding = gpu
    if (N, K) == (2048, 2048):
        W = synth.weights(N, K, "single", n_outlier_cols=4)
        W[::97, 0] += 0.6  # a few blocks with non-zero zero-point
        codes, scales, _ = ref.quantize(W)
        X = synth.activations(M, K, "mm", outlier_frac=0.0 if M == 1 else 0.005)
    else:
        codes, scales = random_packed(N, K, "mm", M, z_fraction=0.02)
        X = synth.activations(M, K, "mm", N)
    assert run_matmul(torch, binding, ref, codes, scales, N, K, X) <= MATMUL_TOL


@pytest.mark.parametrize("M,N,K", [(40, 100, 256), (17, 48, 512), (64, 256, 1024), (130, 1000, 768), (200, 144, 2048), (512, 384, 4096), (129, 257, 1280)])
def test_matmul_tiled_path(gpu, ref, M, N, K):
    torch, binding = gpu
    codes, scales = random_packed(N, K, "gemm", M, z_fraction=0.02)
    X = synth.activations(M, K, "gemm", N)
    assert run_matmul(torch, binding, ref, codes, scales, N, K, X) <= MATMUL_TOL


def test_matmul_quantized_weights_tiled_path(gpu, ref):
    torch, binding = gpu
    N, K, M = 512, 2048, 96
    W = synth.weights(N, K, "gemmq")
    W[::31, 256] -= 0.8
    codes, scales, _ = ref.quantize(W)
    X = synth.activations(M, K, "gemmq")
    assert run_matmul(torch, binding, ref, codes, scales, N, K, X) <= MATMUL_TOL
    # and the product really approximates the unquantized one at 3-bit accuracy (sanity, loose)
    cd, sd = to_dev(torch, codes.view(np.int32)), to_dev(torch, scales.view(np.int32))
    Y = binding.itq3s_matmul(cd, sd, N, K, to_dev(torch, X)).cpu().numpy().astype(np.float64)
    exact = X.astype(np.float64) @ W.astype(np.float64).T
    assert np.linalg.norm(Y - exact) / np.linalg.norm(exact) < 0.6


@pytest.mark.parametrize("M", [1, 16, 40])
def test_matmul_fp16_output_and_strides(gpu, ref, M):
    torch, binding = gpu
    N, K = 304, 1024
    codes, scales = random_packed(N, K, "f16out", M)
    X = synth.activations(M, K, "f16out")
    cd, sd = to_dev(torch, codes.view(np.int32)), to_dev(torch, scales.view(np.int32))
    xbuf = torch.zeros((M, K + 16), dtype=torch.float16, device="cuda")
    xbuf[:, :K] = to_dev(torch, X)
    ybuf = torch.full((M, N + 5), 7.0, dtype=torch.float16, device="cuda")
    binding.itq3s_matmul(cd, sd, N, K, xbuf[:, :K], out=ybuf[:, :N])
    got = ybuf.float().cpu().numpy()
    assert np.all(got[:, N:] == 7.0)
    want = ref.matmul(codes, scales, N, K, X)
    assert rel_rows(got[:, :N], want) <= MATMUL_TOL


def test_matmul_is_deterministic(gpu, ref):
    torch, binding = gpu
    N, K = 4096, 4096
    codes, scales = random_packed(N, K, "det")
    cd, sd = to_dev(torch, codes.view(np.int32)), to_dev(torch, scales.view(np.int32))
    for M in (1, 8, 64):
        X = to_dev(torch, synth.activations(M, K, "det"))
        a = binding.itq3s_matmul(cd, sd, N, K, X).cpu().numpy()
        b = binding.itq3s_matmul(cd, sd, N, K, X).cpu().numpy()
        assert np.array_equal(a, b)


@pytest.mark.parametrize("M,N,K", [(1, 4096, 4096), (4, 1000, 11008), (16, 2048, 2048), (64, 512, 1024)])
def test_matmul_timed_variant_same_result_and_positive_time(gpu, ref, M, N, K):
    """The measurement entry point runs the same kernels: identical output, a plausible duration,
    and a plain call afterwards is unaffected (the armed events are consumed)."""
    torch, binding = gpu
    codes, scales = random_packed(N, K, "timed")
    cd, sd = to_dev(torch, codes.view(np.int32)), to_dev(torch, scales.view(np.int32))
    X = to_dev(torch, synth.activations(M, K, "timed"))
    want = binding.itq3s_matmul(cd, sd, N, K, X).cpu().numpy()
    got, ms = binding.itq3s_matmul_timed(cd, sd, N, K, X)
    assert np.array_equal(got.cpu().numpy(), want)
    assert 0.0 < ms < 50.0
    again = binding.itq3s_matmul(cd, sd, N, K, X).cpu().numpy()
    assert np.array_equal(again, want)


GROUPS = [
    # (K, [N_t], Ms): the projections of a layer that read the same input
    (4096, [4096, 4096, 4096], (1, 4)),          # 7B query / key / value
    (4096, [11008, 11008], (1, 8)),              # 7B gate / up
    (8192, [8192, 1024, 1024], (1, 2, 16)),      # 70B query / key / value (grouped-query attention)
    (11008, [4096, 40], (1, 3)),                 # long K (rotation launch for M = 3), a tensor with 3 row tiles
    (512, [16, 1000, 17, 300], (1, 5)),          # four ragged tensors, one with a single row tile
    (1024, [200, 48], (33,)),                    # tiled path
    (2048, [300, 48, 1000], (20, 32, 300)),      # two passes of the streaming kernel; tiled path with split K and without
    (8192, [12304, 12304], (1,)),                # many row tiles per compute unit, the launch shape of 70B gate / up
    (8192, [8192, 1024, 1024], (1,)),            # the q + k + v launch of the 70B step, as the benchmark launches it
    (8192, [28672, 28672], (1,)),                # its gate + up launch
    (512, [5000, 4100], (2, 8, 16)),             # 570 row tiles: workgroups of two and three tiles, two row sub-groups for M >= 5
    (768, [9000], (5, 16)),                      # 563 row tiles, one tensor, ragged last tile
]


@pytest.mark.parametrize("K,Ns,Ms", GROUPS)
def test_matmul_grouped_matches_oracle_and_single_calls(gpu, ref, K, Ns, Ms):
    """One grouped call = the separate calls, bit for bit (same kernels, same order of sums), and
    within tolerance of the oracle; full rows for the small tensors, sampled rows for the large."""
    torch, binding = gpu
    packed = [random_packed(N, K, "grp", i) for i, N in enumerate(Ns)]
    dev = [(to_dev(torch, c.view(np.int32)), to_dev(torch, s.view(np.int32)), N) for (c, s), N in zip(packed, Ns)]
    rng = np.random.default_rng(5)
    for M in Ms:
        X = synth.activations(M, K, "grp", M)
        Xd = to_dev(torch, X)
        for dtype in (torch.float32, torch.float16):
            outs = binding.itq3s_matmul_grouped(dev, K, Xd, dtype=dtype)
            torch.cuda.synchronize()
            for (c, s), (cd, sd, N), out in zip(packed, dev, outs):
                single = binding.itq3s_matmul(cd, sd, N, K, Xd, dtype=dtype)
                assert torch.equal(out, single)
                if dtype == torch.float32:
                    if N <= 1024:
                        spans = [(0, N)]
                    else:
                        n0 = int(rng.integers(1, N - 600))
                        spans = [(0, 200), (n0, n0 + 200), (N - 200, N)]
                    got = out.cpu().numpy()
                    for n0, n1 in spans:
                        want = ref.matmul(c, s, N, K, X, rows=(n0, n1))
                        assert rel_rows(got[:, n0:n1], want[:, n0:n1]) <= MATMUL_TOL


def test_matmul_grouped_rejects_bad_arguments(gpu, ref):
    torch, binding = gpu
    K = 512
    c, s = random_packed(32, K, "grp-bad")
    dev = (to_dev(torch, c.view(np.int32)), to_dev(torch, s.view(np.int32)), 32)
    X = to_dev(torch, synth.activations(1, K, "grp-bad"))
    with pytest.raises(binding.Itq3sError):
        binding.itq3s_matmul_grouped([dev] * 5, K, X)
    with pytest.raises(binding.Itq3sError):
        binding.itq3s_matmul_grouped([], K, X)
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.Itq3sError, match="workspace"):
        binding.itq3s_matmul_grouped([dev], K, X, workspace=small)


@pytest.mark.parametrize("M", [1, 4, 16, 40, 300])
def test_matmul_extreme_zero_points(gpu, ref, M):
    """Zero-points over the whole stored range (+-2048), on every path: every kernel forms the
    zero-point term in fp32 from the activations themselves."""
    torch, binding = gpu
    N, K = 600, 1024
    codes, scales = random_packed(N, K, "bigz")
    rng = np.random.default_rng(11)
    z = np.zeros(scales.size, dtype=np.float16)
    pick = rng.random(scales.size) < 0.05
    z[pick] = rng.choice(np.array([-2048, -1500, -1024, -1023, -37, 5, 1022, 1023, 1024, 1500, 2047, 2048], dtype=np.float16), size=int(pick.sum()))
    scales = (scales & np.uint32(0xffff)) | (z.view(np.uint16).astype(np.uint32) << np.uint32(16))
    cd, sd = to_dev(torch, codes.view(np.int32)), to_dev(torch, scales.view(np.int32))
    X = synth.activations(M, K, "bigz", M)
    got = binding.itq3s_matmul(cd, sd, N, K, to_dev(torch, X)).cpu().numpy()
    want = ref.matmul(codes, scales, N, K, X)
    assert rel_rows(got, want) <= MATMUL_TOL


@pytest.mark.parametrize("M,N,K", [(2048, 4096, 512), (2000, 4100, 768)])
def test_matmul_large_tile_kernel_ragged_and_zero_points(gpu, ref, M, N, K):
    """Enough 256 x 256 tiles for the large-M kernel; ragged M and N; zero-points over the whole range;
    checked on column spans (first, one that straddles a tile edge, last) for all rows."""
    torch, binding = gpu
    codes, scales = random_packed(N, K, "bigtile")
    rng = np.random.default_rng(12)
    z = np.zeros(scales.size, dtype=np.float16)
    pick = rng.random(scales.size) < 0.02
    z[pick] = rng.choice(np.array([-2048, -1024, -3, 2, 1023, 1024, 2048], dtype=np.float16), size=int(pick.sum()))
    scales = (scales & np.uint32(0xffff)) | (z.view(np.uint16).astype(np.uint32) << np.uint32(16))
    cd, sd = to_dev(torch, codes.view(np.int32)), to_dev(torch, scales.view(np.int32))
    X = synth.activations(M, K, "bigtile", M)
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    got = binding.itq3s_matmul(cd, sd, N, K, to_dev(torch, X), status_flags=flags).cpu().numpy()
    assert int(flags.item()) == 0
    for n0, n1 in [(0, 48), (240, 272), (N - 40, N)]:
        want = ref.matmul(codes, scales, N, K, X, rows=(n0, n1))
        assert rel_rows(got[:, n0:n1], want[:, n0:n1]) <= MATMUL_TOL


def test_matmul_streaming_more_row_tiles_than_one_round(gpu, ref):
    """N large enough that a workgroup per CU would need more than 7 row tiles: the grid grows beyond
    the CU count (a second round); checked on spans at both ends and in the middle."""
    torch, binding = gpu
    N, K = 30000, 512
    codes, scales = random_packed(N, K, "tall")
    cd, sd = to_dev(torch, codes.view(np.int32)), to_dev(torch, scales.view(np.int32))
    for M in (1, 3, 16):
        X = synth.activations(M, K, "tall", M)
        got = binding.itq3s_matmul(cd, sd, N, K, to_dev(torch, X)).cpu().numpy()
        for n0, n1 in [(0, 300), (14990, 15300), (N - 300, N)]:
            want = ref.matmul(codes, scales, N, K, X, rows=(n0, n1))
            assert rel_rows(got[:, n0:n1], want[:, n0:n1]) <= MATMUL_TOL


@pytest.mark.parametrize("scale", [1e-3, 1.0, 200.0])
def test_matmul_activation_magnitudes(gpu, ref, scale):
    """Activations from 1e-3 to several thousand (the rotation keeps its intermediate inside fp16 for
    |x| up to 16376): same relative accuracy on the streaming and the tiled path."""
    torch, binding = gpu
    N, K = 512, 2048
    codes, scales = random_packed(N, K, "mag")
    cd, sd = to_dev(torch, codes.view(np.int32)), to_dev(torch, scales.view(np.int32))
    for M in (1, 4, 8, 48):
        X = (synth.activations(M, K, "mag", M).astype(np.float32) * scale).astype(np.float16)
        assert np.isfinite(X).all()
        got = binding.itq3s_matmul(cd, sd, N, K, to_dev(torch, X)).cpu().numpy()
        want = ref.matmul(codes, scales, N, K, X)
        assert np.isfinite(got).all()
        assert rel_rows(got, want) <= MATMUL_TOL


@pytest.mark.parametrize("M", [1, 3, 8, 16, 40])  # in-kernel rotation, rotation launch + streaming kernel, tiled path
def test_matmul_activation_range_edge_and_flag(gpu, ref, M):
    """The stated activation domain (max|x| <= 16376 and |H x| <= 65504 per 256-channel chunk): at
    its edge the product is finite and matches the oracle with the flag clear; beyond it the library
    says so through ITQ3S_FLAG_ACT_RANGE instead of handing back Inf/NaN silently."""
    torch, binding = gpu
    N, K = 96, 1024
    codes, scales = random_packed(N, K, "range")
    cd, sd = to_dev(torch, codes.view(np.int32)), to_dev(torch, scales.view(np.int32))
    base = synth.activations(M, K, "range", M)

    def run(X):
        flags = torch.zeros(1, dtype=torch.int32, device="cuda")
        Y = binding.itq3s_matmul(cd, sd, N, K, to_dev(torch, X), status_flags=flags).cpu().numpy()
        return Y, int(flags.item())

    # (a) sixteen neighbouring channels (one row of the chunk seen as 16 x 16) at the largest allowed
    # magnitude: the intermediate is exactly 65504
    X = base.copy()
    X[:, 288:304] = np.float16(16376.0)
    X[M - 1, 768:784] = np.float16(-16376.0)
    Y, f = run(X)
    assert f == 0 and np.isfinite(Y).all()
    assert rel_rows(Y, ref.matmul(codes, scales, N, K, X)) <= MATMUL_TOL
    # (b) a whole chunk of +4094: the first rotated value is exactly 65504, the others 0
    X = base.copy()
    X[0, 256:512] = np.float16(4094.0)
    Y, f = run(X)
    assert f == 0 and np.isfinite(Y).all()
    assert rel_rows(Y, ref.matmul(codes, scales, N, K, X)) <= MATMUL_TOL
    # (c) the intermediate overflows (16 * 16400 / 4 rounds to infinity in fp16)
    X = base.copy()
    X[M - 1, 16:32] = np.float16(16400.0)
    Y, f = run(X)
    assert f & binding.FLAG_ACT_RANGE
    # (d) the rotated value overflows (256 * 4100 / 16 > 65504), the intermediate does not
    X = base.copy()
    X[0, 512:768] = np.float16(4100.0)
    Y, f = run(X)
    assert f & binding.FLAG_ACT_RANGE
    # rows that stay inside the domain are unaffected by a row that does not
    if M > 1:
        want = ref.matmul(codes, scales, N, K, X)
        assert rel_rows(Y[1:], want[1:]) <= MATMUL_TOL


def test_matmul_grouped_tiled_path_splits_by_shape_only(gpu, ref):
    """M > 16 with one tensor above 128 output tiles (never split) and one far below (split over K)
    in the same group: each gets exactly what a single call gives it (bit for bit), whatever the
    other tensors are, and a workspace that is too small for the tensor that splits is refused."""
    torch, binding = gpu
    K, M = 2048, 300
    Ns = [11008, 600]  # 3 x 43 = 129 tiles; 3 x 3 = 9 tiles
    packed = [random_packed(N, K, "grp-split", i) for i, N in enumerate(Ns)]
    dev = [(to_dev(torch, c.view(np.int32)), to_dev(torch, s.view(np.int32)), N) for (c, s), N in zip(packed, Ns)]
    X = synth.activations(M, K, "grp-split")
    Xd = to_dev(torch, X)
    need = [binding.itq3s_matmul_workspace_bytes(M, N, K) for N in Ns]
    assert need[1] > need[0]  # the small tensor asks for room for its shares
    outs = binding.itq3s_matmul_grouped(dev, K, Xd)
    singles = [binding.itq3s_matmul(c, s, N, K, Xd) for c, s, N in dev]
    for o, single, (c, s), N in zip(outs, singles, packed, Ns):
        assert torch.equal(o, single)
        for n0, n1 in [(0, 24), (N - 24, N)]:
            want = ref.matmul(c, s, N, K, X, rows=(n0, n1))[:, n0:n1]
            assert rel_rows(o.cpu().numpy()[:, n0:n1], want) <= MATMUL_TOL
    small = torch.empty(need[0], dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.Itq3sError, match="workspace"):
        binding.itq3s_matmul_grouped(dev, K, Xd, workspace=small)


def test_matmul_workspace_shared_by_back_to_back_calls(gpu, ref):
    """One workspace, calls of different shapes and paths enqueued back to back on one stream with no
    host synchronisation in between: each result equals the one computed alone."""
    torch, binding = gpu
    cases = [(1, 1000, 11008), (8, 272, 4096), (40, 512, 1024), (3, 4096, 11008), (1, 2048, 2048)]
    packed = {}
    for M, N, K in cases:
        c, s = random_packed(N, K, "ws")
        packed[(N, K)] = (to_dev(torch, c.view(np.int32)), to_dev(torch, s.view(np.int32)))
    xs = [to_dev(torch, synth.activations(M, K, "ws", i)) for i, (M, N, K) in enumerate(cases)]
    alone = [binding.itq3s_matmul(*packed[(N, K)], N, K, x) for (M, N, K), x in zip(cases, xs)]
    torch.cuda.synchronize()
    ws = torch.empty(max(binding.itq3s_matmul_workspace_bytes(M, N, K) for M, N, K in cases), dtype=torch.uint8, device="cuda")
    for _ in range(3):
        outs = [binding.itq3s_matmul(*packed[(N, K)], N, K, x, workspace=ws) for (M, N, K), x in zip(cases, xs)]
        torch.cuda.synchronize()
        for a, b in zip(alone, outs):
            assert torch.equal(a, b)


@pytest.mark.parametrize("M,N,K", [(129, 100, 8192), (200, 300, 4096), (40, 100, 8192), (8, 100, 8192)])
def test_matmul_fp16_output_with_zero_points_in_most_blocks(gpu, ref, M, N, K):
    """Rows whose blocks nearly all carry a zero-point (a constant offset in the weights), fp16 output: the
    zero-point terms must be applied before the output is rounded -- subtracting them from an already
    rounded fp16 value costs up to 2^-11 of the much larger uncorrected sum (3e-3 of a row was seen)."""
    torch, binding = gpu
    codes, scales = random_packed(N, K, "zp16", M, z_fraction=0.9)
    cd, sd = to_dev(torch, codes.view(np.int32)), to_dev(torch, scales.view(np.int32))
    X = synth.activations(M, K, "zp16", N)
    want = ref.matmul(codes, scales, N, K, X)
    for dtype in (torch.float16, torch.float32):
        got = binding.itq3s_matmul(cd, sd, N, K, to_dev(torch, X), dtype=dtype).cpu().numpy()
        assert rel_rows(got, want) <= (1e-3 if dtype == torch.float16 else 6e-4)


def test_calls_captured_in_a_graph_replay_like_eager(gpu, ref):
    """Every entry point, on every path of the matmul (in-kernel rotation, rotation launch, two passes,
    tiled with and without split-K, grouped), captured once into a HIP graph; between replays the outputs
    and the workspace are overwritten with garbage and eager work runs; every replay must reproduce the
    eager results bit for bit (nothing may depend on state a previous replay left behind)."""
    torch, binding = gpu
    K = 2048
    cases = [(1, 272, K), (16, 100, 36864), (20, 300, K), (200, 300, K), (300, 2100, 512)]
    packed, xs = [], []
    for i, (M, N, Kc) in enumerate(cases):
        c, s = random_packed(N, Kc, "graph", i, z_fraction=0.02)
        packed.append((to_dev(torch, c.view(np.int32)), to_dev(torch, s.view(np.int32))))
        xs.append(to_dev(torch, synth.activations(M, Kc, "graph", i)))
    group = [(packed[0][0], packed[0][1], 272), (packed[2][0], packed[2][1], 300)]
    Wq = to_dev(torch, synth.weights(64, 512, "graph"))
    ws = torch.empty(max(binding.itq3s_matmul_workspace_bytes(M, N, Kc) for M, N, Kc in cases), dtype=torch.uint8, device="cuda")
    outs = [torch.empty((M, N), dtype=torch.float32, device="cuda") for M, N, Kc in cases]
    gouts = [torch.empty((3, n), dtype=torch.float16, device="cuda") for n in (272, 300)]
    qc = torch.empty(binding.itq3s_codes_bytes(64, 512) // 4, dtype=torch.int32, device="cuda")
    qs = torch.empty(binding.itq3s_scales_bytes(64, 512) // 4, dtype=torch.int32, device="cuda")
    deq = torch.empty((272, K), dtype=torch.float32, device="cuda")
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")

    def enqueue():
        for (M, N, Kc), p, x, o in zip(cases, packed, xs, outs):
            binding.itq3s_matmul(*p, N, Kc, x, out=o, workspace=ws, status_flags=flags)
        binding.itq3s_matmul_grouped(group, K, xs[2][:3], outs=gouts, workspace=ws)
        binding.itq3s_quantize(Wq, codes=qc, scales=qs, status_flags=flags)
        binding.itq3s_dequantize(*packed[0], 272, K, out=deq, status_flags=flags)

    results = lambda: [t.clone() for t in outs + gouts + [qc, qs, deq, flags]]
    enqueue()
    torch.cuda.synchronize()
    eager = results()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        enqueue()
    for rep in range(3):
        for t in outs + gouts + [deq]:
            t.fill_(float("nan"))
        qc.fill_(-1)
        qs.fill_(-1)
        ws.fill_(0xA5 + rep)
        torch.cuda.synchronize()
        g.replay()
        # eager work of the program between the replays
        binding.itq3s_matmul(*packed[0], 272, K, xs[0])
        torch.cuda.synchronize()
        for a, b in zip(eager, results()):
            assert torch.equal(a, b), rep


def test_matmul_from_two_host_threads(gpu, ref):
    """Two host threads call the library at the same time, each with its own workspace and outputs
    (streaming, two-pass and tiled shapes, one thread through the timed entry point): every result
    equals the one computed alone, bit for bit."""
    import threading

    torch, binding = gpu
    cases = [(1, 1000, 4096), (8, 272, 4096), (20, 512, 1024), (200, 300, 2048), (3, 4096, 11008)]
    packed, xs = [], []
    for i, (M, N, K) in enumerate(cases):
        c, s = random_packed(N, K, "threads", i)
        packed.append((to_dev(torch, c.view(np.int32)), to_dev(torch, s.view(np.int32))))
        xs.append(to_dev(torch, synth.activations(M, K, "threads", i)))
    alone = [binding.itq3s_matmul(*p, N, K, x) for (M, N, K), p, x in zip(cases, packed, xs)]
    torch.cuda.synchronize()
    errors = []

    def worker(timed):
        try:
            torch.cuda.set_device(0)
            ws = torch.empty(max(binding.itq3s_matmul_workspace_bytes(M, N, K) for M, N, K in cases), dtype=torch.uint8, device="cuda")
            for _ in range(10):
                outs = []
                for (M, N, K), p, x in zip(cases, packed, xs):
                    if timed:
                        y, ms = binding.itq3s_matmul_timed(*p, N, K, x, workspace=ws)
                        assert ms > 0.0
                    else:
                        y = binding.itq3s_matmul(*p, N, K, x, workspace=ws)
                    outs.append(y)
                torch.cuda.synchronize()
                for a, b in zip(alone, outs):
                    assert torch.equal(a, b)
        except BaseException as e:  # reported by the main thread
            errors.append(repr(e))

    threads = [threading.Thread(target=worker, args=(t,)) for t in (False, True)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors


@pytest.mark.parametrize("M,N,K", [(40, 300, 4096), (512, 384, 4096), (200, 1000, 8192), (300, 256, 2048), (1024, 512, 2048)])
def test_matmul_few_tiles_long_k(gpu, ref, M, N, K):
    """Few output tiles and a long K.  The workspace arrives full of garbage, is used three times in a
    row without clearing, and every result equals the first bit for bit and the oracle within
    tolerance; one block in a hundred has a zero-point."""
    torch, binding = gpu
    codes, scales = random_packed(N, K, "fewtiles", M, z_fraction=0.01)
    cd, sd = to_dev(torch, codes.view(np.int32)), to_dev(torch, scales.view(np.int32))
    X = synth.activations(M, K, "fewtiles", N)
    Xd = to_dev(torch, X)
    ws = torch.randint(0, 255, (binding.itq3s_matmul_workspace_bytes(M, N, K),), dtype=torch.uint8, device="cuda")
    first = binding.itq3s_matmul(cd, sd, N, K, Xd, workspace=ws).clone()
    for _ in range(2):
        again = binding.itq3s_matmul(cd, sd, N, K, Xd, workspace=ws)
        assert torch.equal(first, again)
    half = binding.itq3s_matmul(cd, sd, N, K, Xd, dtype=torch.float16, workspace=ws)
    torch.cuda.synchronize()
    want = ref.matmul(codes, scales, N, K, X)
    assert rel_rows(first.cpu().numpy(), want) <= MATMUL_TOL
    assert rel_rows(half.cpu().numpy().astype(np.float64), want) <= MATMUL_TOL


def test_matmul_tiled_shapes_share_a_workspace(gpu, ref):
    """Tiled-path shapes with different tile counts follow each other on the same workspace with no
    host synchronisation in between."""
    torch, binding = gpu
    cases = [(512, 384, 4096), (64, 2048, 1024), (300, 256, 2048), (17, 4096, 4096), (1024, 512, 2048), (512, 384, 4096)]
    packed, xs = [], []
    for i, (M, N, K) in enumerate(cases):
        c, s = random_packed(N, K, "tiled-ws", i)
        packed.append((to_dev(torch, c.view(np.int32)), to_dev(torch, s.view(np.int32))))
        xs.append(to_dev(torch, synth.activations(M, K, "tiled-ws", i)))
    alone = [binding.itq3s_matmul(*pk, N, K, x) for (M, N, K), pk, x in zip(cases, packed, xs)]
    torch.cuda.synchronize()
    ws = torch.randint(0, 255, (max(binding.itq3s_matmul_workspace_bytes(M, N, K) for M, N, K in cases),), dtype=torch.uint8, device="cuda")
    for _ in range(2):
        outs = [binding.itq3s_matmul(*pk, N, K, x, workspace=ws) for (M, N, K), pk, x in zip(cases, packed, xs)]
        torch.cuda.synchronize()
        for a, b in zip(alone, outs):
            assert torch.equal(a, b)


def test_matmul_grouped_flags_and_determinism(gpu, ref):
    """The high-plane check covers every tensor of a grouped call; two identical calls give identical bits."""
    torch, binding = gpu
    K, Ns = 2048, [300, 4096, 48]
    packed = [random_packed(N, K, "grpflag", i) for i, N in enumerate(Ns)]
    bad = packed[2][0].copy()
    bad[(2 * (K // 256) + 1) * 384 + 256 + 7] |= np.uint32(1 << 9)  # a high-plane bit in the last tensor
    X = to_dev(torch, synth.activations(2, K, "grpflag"))
    for variant, expect in ((packed[2][0], 0), (bad, 8)):
        dev = [(to_dev(torch, c.view(np.int32)), to_dev(torch, s.view(np.int32)), N) for (c, s), N in zip(packed[:2] + [(variant, packed[2][1])], Ns)]
        flags = torch.zeros(1, dtype=torch.int32, device="cuda")
        a = binding.itq3s_matmul_grouped(dev, K, X, status_flags=flags)
        b = binding.itq3s_matmul_grouped(dev, K, X)
        torch.cuda.synchronize()
        assert int(flags.item()) == expect
        for u, v in zip(a, b):
            assert torch.equal(u, v)


@pytest.mark.parametrize("M,N,K", [(1, 48, 512), (17, 1000, 768), (130, 144, 2048), (300, 600, 1024), (512, 384, 4096), (700, 200, 512), (1030, 136, 768)])
def test_matmul_weight_side_matches_oracle(gpu, ref, M, N, K):
    """The paper's placement of the transform (inside the weight tile loader): same product, same bar;
    zero-points over the whole range are exact here (they only touch channel 0 of a block)."""
    torch, binding = gpu
    codes, scales = random_packed(N, K, "ws-side", z_fraction=0.02)
    rng = np.random.default_rng(13)
    z = (scales >> np.uint32(16)).astype(np.uint16).view(np.float16).copy()
    pick = rng.random(scales.size) < 0.01
    z[pick] = rng.choice(np.array([-2048, -1000, 1023, 2048], dtype=np.float16), size=int(pick.sum()))
    scales = (scales & np.uint32(0xffff)) | (z.view(np.uint16).astype(np.uint32) << np.uint32(16))
    cd, sd = to_dev(torch, codes.view(np.int32)), to_dev(torch, scales.view(np.int32))
    X = synth.activations(M, K, "ws-side", M)
    want = ref.matmul(codes, scales, N, K, X)
    for dtype in (torch.float32, torch.float16):
        flags = torch.zeros(1, dtype=torch.int32, device="cuda")
        got = binding.itq3s_matmul_weight_side(cd, sd, N, K, to_dev(torch, X), dtype=dtype, status_flags=flags).cpu().numpy()
        assert int(flags.item()) == 0
        assert rel_rows(got, want) <= MATMUL_TOL


def test_matmul_weight_side_full_size_sampled(gpu, ref):
    torch, binding = gpu
    N, K, M = 14336, 4096, 512
    W = synth.weights(N, K, "prefill-ws")
    codes, scales = binding.itq3s_quantize(to_dev(torch, W))
    hc, hs = u32(codes), u32(scales)
    X = synth.activations(M, K, "prefill-ws")
    got, ms = binding.itq3s_matmul_weight_side(codes, scales, N, K, to_dev(torch, X), timed=True)
    assert ms > 0.0
    got = got.cpu().numpy()
    for n0, n1 in [(0, 40), (7000, 7040), (N - 40, N)]:
        want = ref.matmul(hc, hs, N, K, X, rows=(n0, n1))
        assert rel_rows(got[:, n0:n1], want[:, n0:n1]) <= MATMUL_TOL


def test_matmul_flags_high_plane(gpu, ref):
    torch, binding = gpu
    codes, scales = random_packed(64, 512, "hp")
    bad = codes.copy()
    bad[384 * 3 + 256 + 77] |= np.uint32(1 << 20)
    for M in (1, 32):
        flags = torch.zeros(1, dtype=torch.int32, device="cuda")
        binding.itq3s_matmul(to_dev(torch, bad.view(np.int32)), to_dev(torch, scales.view(np.int32)), 64, 512,
                             to_dev(torch, synth.activations(M, 512, "hp")), status_flags=flags)
        assert int(flags.item()) == binding.FLAG_BAD_CODE
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    binding.itq3s_matmul_weight_side(to_dev(torch, bad.view(np.int32)), to_dev(torch, scales.view(np.int32)), 64, 512,
                                     to_dev(torch, synth.activations(32, 512, "hp")), status_flags=flags)
    assert int(flags.item()) == binding.FLAG_BAD_CODE


def sample_row_ranges(N, count, seed):
    rng = np.random.default_rng(seed)
    starts = sorted(set([0, max(N - 16, 0)] + [int(v) for v in rng.integers(0, max(N - 16, 1), size=count)]))
    return [(s, min(s + 16, N)) for s in starts]


FULL = [
    ("llama7b", 4096, 4096, (1, 8)),
    ("llama7b", 11008, 4096, (1, 8)),
    ("llama7b", 4096, 11008, (1, 4, 8)),
    ("llama70b", 8192, 8192, (1, 4, 16)),
    ("llama70b", 28672, 8192, (1, 4, 16)),
    ("llama70b", 8192, 28672, (1, 2, 16)),
    ("llama70b", 1024, 8192, (1, 4, 16)),
]


@pytest.mark.parametrize("name,N,K,Ms", FULL)
def test_matmul_full_size_sampled_rows(gpu, ref, name, N, K, Ms):
    """The benchmark's shapes in the benchmark's launch configuration; the oracle recomputes a
    sample of 16-row ranges (first, last and random ones) for every activation row."""
    torch, binding = gpu
    codes, scales = random_packed(N, K, name, z_fraction=0.001)
    for M in Ms:
        X = synth.activations(M, K, name, N)
        worst = run_matmul(torch, binding, ref, codes, scales, N, K, X, rows=sample_row_ranges(N, 6, N + K + M))
        assert worst <= MATMUL_TOL, (N, K, M, worst)


@pytest.mark.parametrize("N,K,M", [(14336, 4096, 512), (4096, 14336, 512), (14336, 4096, 2048), (4096, 4096, 2048), (3700, 512, 1100), (4100, 768, 1000)])
def test_matmul_prefill_full_size_sampled(gpu, ref, N, K, M):
    """The benchmark's prefill shapes and a few with 129..256 tiles (one workgroup per compute unit):
    sampled activation rows and weight-row ranges against the oracle, first and last tile included."""
    torch, binding = gpu
    codes, scales = random_packed(N, K, "prefill", z_fraction=0.001)
    X = synth.activations(M, K, "prefill", N)
    cd, sd = to_dev(torch, codes.view(np.int32)), to_dev(torch, scales.view(np.int32))
    Y = binding.itq3s_matmul(cd, sd, N, K, to_dev(torch, X), dtype=torch.float16)
    torch.cuda.synchronize()
    Y = Y.float().cpu().numpy()
    rng = np.random.default_rng(N + M)
    msel = np.unique(np.concatenate([[0, M - 1], rng.integers(0, M, 14)]))
    worst = 0.0
    for n0, n1 in sample_row_ranges(N, 10, N + K):
        want = ref.matmul(codes, scales, N, K, X[msel], rows=(n0, n1))[:, n0:n1]
        worst = max(worst, np.max(np.linalg.norm(Y[msel][:, n0:n1] - want, axis=1) / np.linalg.norm(want, axis=1)))
    assert worst <= MATMUL_TOL


def test_end_to_end_config1(gpu, ref):
    """Config 1 as one pipeline on the GPU: quantize -> matmul, against oracle quantize -> matmul."""
    torch, binding = gpu
    N = K = 2048
    W = synth.weights(N, K, "single", n_outlier_cols=4)
    X = synth.activations(1, K, "single", outlier_frac=0.0)
    codes, scales = binding.itq3s_quantize(to_dev(torch, W))
    Y = binding.itq3s_matmul(codes, scales, N, K, to_dev(torch, X)).cpu().numpy()
    rc, rs, _ = ref.quantize(W)
    assert np.array_equal(u32(codes), rc) and np.array_equal(u32(scales), rs)
    assert rel_rows(Y, ref.matmul(rc, rs, N, K, X)) <= MATMUL_TOL
