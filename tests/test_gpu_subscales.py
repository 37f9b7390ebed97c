"""HIP path vs CPU oracle for the sub-block-scale variant of the format (Sec. 4.1: 8 fp16 sub-scales,
116 bytes per block), through the C ABI.  Bars as for the base format: codes, scale words and
sub-scale words bit-exact; dequantize <= 1e-6 relative L2 per row; matmul <= 2e-3 per activation row."""
import numpy as np
import pytest

from paper_2603_27914_amd import synth

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


def u32(t):
    return t.cpu().numpy().view(np.uint32)


def rel_rows(got, want):
    return np.max(np.linalg.norm(got.astype(np.float64) - want, axis=1) / np.maximum(np.linalg.norm(want, axis=1), 1e-300))


def uneven_weights(N, K, *key):
    """Weights whose rotated blocks have sub-blocks of different energy (what the variant is for), a few
    non-zero zero-points, one all-zero block and one block with a quiet sub-block."""
    W = synth.weights(N, K, "sub", *key)
    rng = np.random.default_rng(abs(hash(key)) % (1 << 31))
    k = np.arange(256)
    pc = np.array([bin(v).count("1") for v in range(256)])
    H = (1 - 2 * (pc[k[:, None] & k[None, :]] & 1)).astype(np.float64) / 16.0
    for n in range(0, N, 3):
        b = int(rng.integers(0, K // 256))
        prof = np.repeat(np.exp(rng.normal(size=8)), 32)
        W[n, 256 * b : 256 * b + 256] = (H @ (rng.normal(size=256) * prof * 0.02)).astype(np.float32)
    W[::7, 0] += 0.6
    if N > 5:
        W[5, :256] = 0.0
    return W


@pytest.mark.parametrize("N,K,ldw", [(16, 256, None), (40, 768, None), (333, 1024, 1040), (1000, 2048, None)])
def test_quantize_sub_bit_exact(gpu, ref, N, K, ldw):
    torch, binding = gpu
    W = uneven_weights(N, K, N, K)
    if ldw is None:
        Wd = dev(torch, W)
    else:
        buf = torch.zeros((N, ldw), dtype=torch.float32, device="cuda")
        buf[:, :K] = dev(torch, W)
        Wd = buf[:, :K]
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    codes, scales, subs = binding.itq3s_quantize_sub(Wd, status_flags=flags)
    torch.cuda.synchronize()
    rc, rs, rsub, rflags = ref.quantize_sub(W)
    assert np.array_equal(u32(scales), rs), "scale words differ"
    assert np.array_equal(u32(subs), rsub), "sub-scale words differ"
    assert np.array_equal(u32(codes), rc), "packed codes differ"
    assert int(flags.item()) == rflags
    # the first 100 bytes of every block are those of the base format's quantizer
    c0, s0 = binding.itq3s_quantize(Wd)
    assert torch.equal(s0, scales)


def test_quantize_sub_adversarial_blocks(gpu, ref):
    torch, binding = gpu
    rng = np.random.default_rng(3)
    W = (0.02 * rng.standard_t(4.0, size=(64, 512))).astype(np.float32)
    W[0, :256] = 0.0
    W[1, :256] = 1.0                      # only coefficient 0 is non-zero after rotation
    W[2, 7] = np.inf
    W[3, 300] = np.nan
    W[4, :256] *= 1e-30                   # scale underflows
    W[5, :256] *= 1e30
    W[6, :256] = 3.0e38                   # scale saturates
    W[7, 5] = 1e20                        # one spike: flat spectrum
    Wd = dev(torch, W)
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    codes, scales, subs = binding.itq3s_quantize_sub(Wd, status_flags=flags)
    rc, rs, rsub, rflags = ref.quantize_sub(W)
    assert np.array_equal(u32(scales), rs) and np.array_equal(u32(subs), rsub) and np.array_equal(u32(codes), rc)
    assert int(flags.item()) == rflags


@pytest.mark.parametrize("N,K", [(40, 768), (600, 2048)])
def test_dequantize_sub(gpu, ref, N, K):
    torch, binding = gpu
    W = uneven_weights(N, K, "deq", N)
    rc, rs, rsub, _ = ref.quantize_sub(W)
    cd, sd, ud = dev(torch, rc.view(np.int32)), dev(torch, rs.view(np.int32)), dev(torch, rsub.view(np.int32))
    want = ref.dequantize_sub(rc, rs, rsub, N, K)
    got = binding.itq3s_dequantize_sub(cd, sd, ud, N, K).cpu().numpy()
    assert rel_rows(got, want) <= 1e-6
    assert np.max(np.abs(got - want)) <= 2.0 ** -22 * np.max(np.abs(want)) * 4
    got16 = binding.itq3s_dequantize_sub(cd, sd, ud, N, K, dtype=torch.float16).float().cpu().numpy()
    assert rel_rows(got16, want) <= 1e-3
    # sub-scales 1 everywhere: the base format, bit for bit
    ones = torch.full_like(ud, 0x3C003C00)
    assert torch.equal(binding.itq3s_dequantize_sub(cd, sd, ones, N, K), binding.itq3s_dequantize(cd, sd, N, K))


@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 7, 16, 20, 37, 64])  # fused rotation; rotation launch (8 and 16 padded rows); several passes
@pytest.mark.parametrize("N,K", [(48, 512), (1000, 1024), (1160, 4096), (272, 11008), (9000, 512)])
def test_matmul_sub(gpu, ref, M, N, K):
    torch, binding = gpu
    W = uneven_weights(N, K, "mm", N)
    rc, rs, rsub, _ = ref.quantize_sub(W)
    cd, sd, ud = dev(torch, rc.view(np.int32)), dev(torch, rs.view(np.int32)), dev(torch, rsub.view(np.int32))
    X = synth.activations(M, K, "sub-mm", M, N)
    want = ref.matmul_sub(rc, rs, rsub, N, K, X)
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    for dtype in (torch.float32, torch.float16):
        got = binding.itq3s_matmul_sub(cd, sd, ud, N, K, dev(torch, X), dtype=dtype, status_flags=flags).float().cpu().numpy()
        assert rel_rows(got, want) <= 2e-3
    assert int(flags.item()) == 0
    if M == 3:
        ones = torch.full_like(ud, 0x3C003C00)  # sub-scales 1: the base format's product
        a = binding.itq3s_matmul_sub(cd, sd, ones, N, K, dev(torch, X)).cpu().numpy()
        assert rel_rows(a, ref.matmul(rc, rs, N, K, X)) <= 2e-3


@pytest.mark.parametrize("M,N,K", [(65, 48, 512), (130, 1000, 768), (600, 200, 512), (1030, 136, 1024)])
def test_matmul_sub_many_rows(gpu, ref, M, N, K):
    """Above 64 rows the product runs on the tiled kernel that reconstructs weight tiles on chip (sub-scaled
    digits through the inverse transform, one rounding of w_hat to fp16): same bar; one and several
    512-row slabs, row tiles beyond the tensor, and the base format's product for sub-scales 1."""
    torch, binding = gpu
    W = uneven_weights(N, K, "mm-rows", N)
    rc, rs, rsub, _ = ref.quantize_sub(W)
    cd, sd, ud = dev(torch, rc.view(np.int32)), dev(torch, rs.view(np.int32)), dev(torch, rsub.view(np.int32))
    X = synth.activations(M, K, "sub-rows", M, N)
    want = ref.matmul_sub(rc, rs, rsub, N, K, X)
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    for dtype in (torch.float32, torch.float16):
        got = binding.itq3s_matmul_sub(cd, sd, ud, N, K, dev(torch, X), dtype=dtype, status_flags=flags).float().cpu().numpy()
        assert rel_rows(got, want) <= 2e-3
    assert int(flags.item()) == 0
    ones = torch.full_like(ud, 0x3C003C00)
    a = binding.itq3s_matmul_sub(cd, sd, ones, N, K, dev(torch, X)).cpu().numpy()
    assert rel_rows(a, ref.matmul(rc, rs, N, K, X)) <= 2e-3


def test_matmul_sub_full_size_sampled(gpu, ref):
    """A 70B-shaped tensor in the launch configuration a decode step uses, checked on sampled rows."""
    torch, binding = gpu
    N, K = 8192, 8192
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    W = torch.randn((N, K), generator=gen, device="cuda") * 0.02
    W[:, ::97] *= 8.0
    codes, scales, subs = binding.itq3s_quantize_sub(W)
    X = synth.activations(1, K, "sub-full")
    got = binding.itq3s_matmul_sub(codes, scales, subs, N, K, dev(torch, X)).cpu().numpy()
    hc, hs, hu = u32(codes), u32(scales), u32(subs)
    for n0, n1 in [(0, 32), (4000, 4032), (N - 32, N)]:
        want = ref.matmul_sub(hc, hs, hu, N, K, X, rows=(n0, n1))[:, n0:n1]
        assert rel_rows(got[:, n0:n1], want) <= 2e-3
    # and the packed bytes against the oracle's quantizer on those rows' tiles
    Wh = W[:48].cpu().numpy()
    rc, rs, rsub, _ = ref.quantize_sub(Wh)
    KB = K // 256
    assert np.array_equal(hc[: 3 * KB * 384], rc) and np.array_equal(hs[: 3 * KB * 16], rs) and np.array_equal(hu[: 3 * KB * 64], rsub)


def test_sub_rejects_bad_arguments(gpu):
    torch, binding = gpu
    N, K = 32, 512
    W = torch.zeros((N, K), dtype=torch.float32, device="cuda")
    codes, scales, subs = binding.itq3s_quantize_sub(W)
    X = torch.zeros((2, K), dtype=torch.float16, device="cuda")
    with pytest.raises(binding.Itq3sError, match="subscales"):
        binding.itq3s_matmul_sub(codes, scales, subs[:-1], N, K, X)
    with pytest.raises(binding.Itq3sError, match="subscales"):
        binding.itq3s_dequantize_sub(codes, scales, subs.float(), N, K)
    X8 = torch.zeros((8, K), dtype=torch.float16, device="cuda")
    with pytest.raises(binding.Itq3sError, match="workspace"):
        binding.itq3s_matmul_sub(codes, scales, subs, N, K, X8, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert binding.itq3s_subscales_bytes(N, K) == 2 * 2 * 256 and binding.itq3s_subscales_bytes(N, 500) == 0
