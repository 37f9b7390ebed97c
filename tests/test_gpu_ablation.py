"""Block-size ablation (Sec. 6, "Ablation: FWHT Block Size") on the GPU: itq3s_roundtrip against the
oracle's roundtrip_n for every transform length 32 .. 512.  Needs a real MI355X: -m gpu.

Bars: codes and scale words bit-exact, status flags equal, reconstructed weights <= 1e-6 relative L2
per row (on data in the normal fp32 range they are the oracle's fp64 values rounded once, so equal
bit for bit), error sums to 1e-9 relative (atomic additions in no fixed order)."""
import numpy as np
import pytest

from paper_2603_27914_amd import synth

pytestmark = pytest.mark.gpu

SIZES = [32, 64, 128, 256, 512]
WHAT_TOL = 1e-6


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


def check_roundtrip(torch, binding, ref, W, n, ldw=None, exact=True):
    N, K = W.shape
    if ldw is None:
        Wd = to_dev(torch, W)
    else:
        buf = torch.zeros((N, ldw), dtype=torch.float32, device="cuda")
        buf[:, :K] = to_dev(torch, W)
        Wd = buf[:, :K]
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    err2 = torch.zeros(2, dtype=torch.float64, device="cuda")
    codes, scales, what = binding.itq3s_roundtrip(Wd, n, err2=err2, status_flags=flags)
    torch.cuda.synchronize()
    rc, rs, rw, rflags = ref.roundtrip_n(W, n)
    assert np.array_equal(scales.cpu().numpy().view(np.uint32), rs), "scale words differ (n = %d)" % n
    assert np.array_equal(codes.cpu().numpy(), rc), "codes differ (n = %d)" % n
    assert int(flags.item()) == rflags
    got = what.cpu().numpy()
    num = np.linalg.norm(got.astype(np.float64) - rw, axis=1)
    den = np.linalg.norm(rw, axis=1)
    assert np.all(num <= WHAT_TOL * den + 1e-37), "reconstruction differs (n = %d)" % n
    if exact:
        assert np.array_equal(got, rw.astype(np.float32))
    # error sums over the blocks without non-finite weights, from the oracle's reconstruction
    Wb = W.astype(np.float64).reshape(N, K // n, n)
    fin = np.all(np.isfinite(Wb), axis=2)
    with np.errstate(invalid="ignore", over="ignore"):
        se = np.sum(np.where(fin[:, :, None], (rw.astype(np.float32).astype(np.float64).reshape(N, K // n, n) - Wb) ** 2, 0.0))
        sw = np.sum(np.where(fin[:, :, None], Wb**2, 0.0))
    e = err2.cpu().numpy()
    if np.isfinite(se) and np.isfinite(sw):
        assert abs(e[0] - se) <= 1e-9 * se + 1e-300 and abs(e[1] - sw) <= 1e-9 * sw + 1e-300
    return codes, scales, what


@pytest.mark.parametrize("n", SIZES)
def test_roundtrip_weights_like_the_papers(gpu, ref, n):
    """Heavy-tailed rows with outlier columns; 2048 channels = two wavefront chunks per row."""
    torch, binding = gpu
    check_roundtrip(torch, binding, ref, synth.weights(512, 2048, "abl", n, n_outlier_cols=4), n)


@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("N,K,ldw", [(1, 512, None), (3, 1536, None), (37, 2560, 2564), (130, 4608, None)])
def test_roundtrip_ragged_shapes(gpu, ref, n, N, K, ldw):
    """K not a multiple of the 1024 channels a wavefront covers; padded rows; few rows."""
    torch, binding = gpu
    check_roundtrip(torch, binding, ref, synth.weights(N, K, "abl-ragged", n, N, n_outlier_cols=2), n, ldw)


def adversarial_rows(n, rng):
    from scipy.linalg import hadamard

    rows = []
    rows.append(np.zeros(n, np.float32))  # all zero: scale 0
    rows.append(np.full(n, 0.37, np.float32))  # constant: a spike after the transform, sigma > 0
    e0 = np.zeros(n, np.float32); e0[0] = 3.0; rows.append(e0)  # spike at 0: constant after the transform, sigma = 0
    e5 = np.zeros(n, np.float32); e5[5] = -7.0; rows.append(e5)
    rows.append((rng.standard_normal(n) * 1e6).astype(np.float32))  # scale saturates
    rows.append((rng.standard_normal(n) * 1e-7).astype(np.float32))  # subnormal fp16 scale
    rows.append((rng.standard_normal(n) * 1e-9).astype(np.float32))  # scale underflows to 0
    w = (rng.standard_normal(n) * 1e-3).astype(np.float32); w[0] = 1e3; rows.append(w)  # z clamps
    w = (rng.standard_normal(n) * 1e-5).astype(np.float32) + np.float32(4.0); rows.append(w)  # constant plus noise: a spike after the transform
    w = (0.02 * rng.standard_t(4, n)).astype(np.float32); w[0] = 0.9; rows.append(w)  # z != 0
    w = (0.02 * rng.standard_t(4, n)).astype(np.float32); w[0] = -1.7; rows.append(w)
    w = rng.standard_normal(n).astype(np.float32); w[n // 3] = np.inf; rows.append(w)
    w = rng.standard_normal(n).astype(np.float32); w[n - 1] = np.nan; rows.append(w)
    rows.append((rng.standard_normal(n) * np.finfo(np.float32).tiny).astype(np.float32))
    H = hadamard(n).astype(np.float64)
    for _ in range(10):  # integer-valued transform-domain data
        target = rng.integers(-40, 41, size=n).astype(np.float64) * 16.0
        rows.append((H @ target / n).astype(np.float32))
    return np.stack(rows)


@pytest.mark.parametrize("n", SIZES)
def test_roundtrip_adversarial_blocks(gpu, ref, n):
    torch, binding = gpu
    rng = np.random.default_rng(1000 + n)
    B = adversarial_rows(n, rng)
    # every block type next to every other inside one wavefront: rows of 2048 / n ... blocks
    per_row = max(2, 1024 // n)
    reps = [np.roll(B, s, axis=0) for s in range(per_row)]
    W = np.concatenate(reps, axis=1)
    if W.shape[1] % 32:
        W = np.concatenate([W, W], axis=1)
    check_roundtrip(torch, binding, ref, np.ascontiguousarray(W), n, exact=False)


def test_roundtrip_256_equals_quantize_and_dequantize(gpu, ref):
    """Block size 256 is the packed format's path: same scale words, same codes, same w_hat."""
    torch, binding = gpu
    N, K = 96, 1024
    W = synth.weights(N, K, "abl-256")
    Wd = to_dev(torch, W)
    codes, scales, what = binding.itq3s_roundtrip(Wd, 256)
    pc, ps = binding.itq3s_quantize(Wd)
    deq = binding.itq3s_dequantize(pc, ps, N, K)
    torch.cuda.synchronize()
    assert np.array_equal(what.cpu().numpy(), deq.cpu().numpy())
    s = ps.cpu().numpy().view(np.uint32).reshape(N // 16, K // 256, 16)  # tile (nt, b), row r
    assert np.array_equal(scales.cpu().numpy().view(np.uint32), s.transpose(0, 2, 1).reshape(N, K // 256))
    rc, _, _, _ = ref.roundtrip_n(W, 256)
    assert np.array_equal(codes.cpu().numpy(), rc)


def test_roundtrip_optional_outputs_and_accumulating_sums(gpu, ref):
    torch, binding = gpu
    W = synth.weights(64, 1024, "abl-opt")
    Wd = to_dev(torch, W)
    err2 = torch.zeros(2, dtype=torch.float64, device="cuda")
    c, s, w = binding.itq3s_roundtrip(Wd, 128, codes=False, scales=False, w_hat=False, err2=err2)
    assert c is None and s is None and w is None
    first = err2.cpu().numpy().copy()
    binding.itq3s_roundtrip(Wd, 128, codes=False, scales=False, w_hat=False, err2=err2)
    torch.cuda.synchronize()
    assert np.allclose(err2.cpu().numpy(), 2 * first, rtol=1e-12)
    _, _, rw, _ = ref.roundtrip_n(W, 128)
    assert abs(first[0] - np.sum((rw.astype(np.float32).astype(np.float64) - W) ** 2)) <= 1e-9 * first[0]
    # only the reconstruction, into a padded buffer
    buf = torch.full((64, 1032), 7.0, dtype=torch.float32, device="cuda")
    binding.itq3s_roundtrip(Wd, 128, codes=False, scales=False, w_hat=buf[:, :1024])
    torch.cuda.synchronize()
    assert np.array_equal(buf[:, :1024].cpu().numpy(), rw.astype(np.float32))
    assert bool((buf[:, 1024:] == 7.0).all())


def test_roundtrip_rejects_bad_arguments(gpu, ref):
    torch, binding = gpu
    W = torch.zeros((4, 768), dtype=torch.float32, device="cuda")
    for n in (0, 16, 48, 1024):
        with pytest.raises(binding.Itq3sError):
            binding.itq3s_roundtrip(W, n)
    with pytest.raises(binding.Itq3sError):
        binding.itq3s_roundtrip(W, 512)  # 768 % 512 != 0
    with pytest.raises(binding.Itq3sError):
        binding.itq3s_roundtrip(W[:, 1:513], 256)  # misaligned start
    import ctypes

    L = binding.lib()
    assert L.itq3s_roundtrip(None, 4, 768, 768, 256, None, None, None, 0, None, None, None) == -1
    assert L.itq3s_roundtrip(ctypes.c_void_p(W.data_ptr()), 4, 768, 768, 96, None, None, None, 0, None, None, None) == -2


@pytest.mark.parametrize("n", SIZES)
def test_roundtrip_full_size_sampled(gpu, ref, n):
    """Llama-7B-shaped tensor (4096 x 11008 would not divide by 512; 11008 = 43 * 256): the 4096 x 4096
    attention shape at full size for every n, the oracle on sampled rows."""
    torch, binding = gpu
    N, K = 4096, 4096
    W = synth.weights(N, K, "abl-full")
    Wd = to_dev(torch, W)
    err2 = torch.zeros(2, dtype=torch.float64, device="cuda")
    codes, scales, what = binding.itq3s_roundtrip(Wd, n, err2=err2)
    torch.cuda.synchronize()
    rows = np.random.default_rng(n).choice(N, 48, replace=False)
    rc, rs, rw, _ = ref.roundtrip_n(np.ascontiguousarray(W[rows]), n)
    assert np.array_equal(codes.cpu().numpy()[rows], rc)
    assert np.array_equal(scales.cpu().numpy().view(np.uint32)[rows], rs)
    assert np.array_equal(what.cpu().numpy()[rows], rw.astype(np.float32))
    # the error sums are those of the returned reconstruction
    got = what.cpu().numpy().astype(np.float64)
    e = err2.cpu().numpy()
    assert abs(e[0] - np.sum((got - W) ** 2)) <= 1e-9 * e[0]
    assert abs(e[1] - np.sum(W.astype(np.float64) ** 2)) <= 1e-9 * e[1]
    # Thm 1 (isometry) consequence: the relative error of ternary coding with the optimal scale stays
    # in a narrow band whatever the block size
    assert 0.3 < np.sqrt(e[0] / e[1]) < 0.6
