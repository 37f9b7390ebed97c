"""Host-side checks of the C-ABI library: it loads, exports every symbol the header declares, its
size helpers agree with the format description, and argument errors are reported without
launching anything (these calls return before the first HIP call, so they run without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2603_27914_amd import binding, build

    if not os.path.exists(binding.LIB_PATH):
        build.build_lib()
    return binding.lib()


def declared_functions():
    names = set()
    for header in ("itq3s.h", "itq3s_bench.h"):  # the product interface and the measurement aids
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(itq3s_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_product_header_keeps_its_contract():
    """Nothing that waits for the device is declared in the product header."""
    text = open(os.path.join(ROOT, "include", "itq3s.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    assert "_timed" not in text and "read_probe" not in text and "kernel_ms" not in text


def test_library_exports_every_declared_symbol(L):
    from paper_2603_27914_amd import binding

    names = declared_functions()
    assert len(names) >= 8
    for n in names:
        assert hasattr(L, n), n
    assert sorted(binding.EXPORTS) == names
    for n in names:  # the Python binding carries the same names
        if n != "itq3s_strerror":
            assert hasattr(binding, n), n


def test_size_helpers(L):
    assert L.itq3s_codes_bytes(16, 256) == 1536 and L.itq3s_scales_bytes(16, 256) == 64
    assert L.itq3s_codes_bytes(17, 512) == 2 * 2 * 1536
    assert L.itq3s_codes_bytes(2048, 2048) + L.itq3s_scales_bytes(2048, 2048) == 2048 * 8 * 100
    assert L.itq3s_codes_bytes(16, 255) == 0 and L.itq3s_scales_bytes(0, 256) == 0
    # the 70B-shaped stream: 267,386,880 blocks of 100 bytes
    from paper_2603_27914_amd import synth

    total = sum(c * (L.itq3s_codes_bytes(n, k) + L.itq3s_scales_bytes(n, k)) for _, n, k, c in synth.LLAMA70B_LAYER) * 80
    assert total == 26_738_688_000
    assert L.itq3s_matmul_workspace_bytes(1, 4096, 4096) == 256 and L.itq3s_matmul_workspace_bytes(4, 4096, 28672) == 256
    assert L.itq3s_matmul_workspace_bytes(8, 4096, 4096) >= 8 * 4096 * 2 + 8 * 16 * 8
    assert L.itq3s_matmul_workspace_bytes(512, 4096, 4096) >= 512 * 4096 * 2
    assert L.itq3s_version() >= 100


def test_argument_errors_return_before_any_launch(L):
    buf = (ctypes.c_uint8 * 4096)()
    p = ctypes.cast(buf, ctypes.c_void_p)
    addr = (p.value + 255) & ~255
    ok = ctypes.c_void_p(addr)
    odd = ctypes.c_void_p(addr + 2)
    assert L.itq3s_quantize(None, 16, 256, 256, ok, ok, None, None) == -1
    assert L.itq3s_quantize(ok, 16, 250, 256, ok, ok, None, None) == -2
    assert L.itq3s_quantize(ok, 0, 256, 256, ok, ok, None, None) == -2
    assert L.itq3s_quantize(ok, 16, 256, 128, ok, ok, None, None) == -2
    assert L.itq3s_quantize(odd, 16, 256, 256, ok, ok, None, None) == -3
    assert L.itq3s_quantize(ok, 16, 256, 258, ok, ok, None, None) == -3
    assert L.itq3s_dequantize(ok, ok, 16, 256, ok, 7, 256, None, None) == -4
    assert L.itq3s_dequantize(ok, None, 16, 256, ok, 0, 256, None, None) == -1
    assert L.itq3s_matmul(ok, ok, 16, 256, ok, 1, 256, ok, 0, 16, None, 0, None, None) == -5
    assert L.itq3s_matmul(ok, ok, 16, 256, ok, 1, 256, ok, 0, 16, ok, 8, None, None) == -5
    assert L.itq3s_matmul(ok, ok, 16, 256, ok, 8, 256, ok, 0, 16, ok, 1024, None, None) == -5
    assert L.itq3s_matmul(ok, ok, 16, 1 << 29, ok, 1, 1 << 29, ok, 0, 16, ok, 1 << 20, None, None) == -2
    assert L.itq3s_matmul(ok, ok, 16, 256, ok, 1, 256, ok, 0, 8, ok, 1 << 20, None, None) == -2
    assert L.itq3s_matmul(ok, ok, 16, 256, ok, 1, 250, ok, 0, 16, ok, 1 << 20, None, None) == -2
    assert L.itq3s_matmul(ok, ok, 16, 256, ok, 1, 260, ok, 0, 16, ok, 1 << 20, None, None) == -3
    assert L.itq3s_matmul(ok, ok, 16, 256, ok, 1, 256, ok, 3, 16, ok, 1 << 20, None, None) == -4
    for code in range(0, -7, -1):
        assert len(L.itq3s_strerror(code)) > 0
    assert L.itq3s_strerror(-99) == b"unknown status"


def test_binding_refuses_cpu_tensors():
    import torch

    from paper_2603_27914_amd import binding

    with pytest.raises(binding.Itq3sError):
        binding.itq3s_quantize(torch.zeros(16, 256))


def test_binding_checks_packed_tensors_against_the_shape():
    """The C ABI takes pointers and trusts N and K; the binding refuses tensors that do not hold
    W[N, K] before anything is launched (a kernel reading past them would fault the device)."""
    import torch

    from paper_2603_27914_amd import binding

    N, K = 40, 512
    cw, sw = binding.itq3s_codes_bytes(N, K) // 4, binding.itq3s_scales_bytes(N, K) // 4
    codes, scales = torch.zeros(cw, dtype=torch.int32), torch.zeros(sw, dtype=torch.int32)
    binding._need_packed(codes, scales, N, K)  # fits
    binding._need_packed(codes, scales, 33, K)  # same number of row tiles
    for bad_args, what in [
        ((codes, scales, 64, K), "holds"),                      # more rows than stored
        ((codes, scales, N, 1024), "holds"),                    # longer rows than stored
        ((codes[:-1], scales, N, K), "holds"),                  # a tensor cut short
        ((codes, scales[: sw // 2], N, K), "holds"),
        ((codes, scales, N, 500), "bad shape"),                 # K not a multiple of 256
        ((codes, scales, 0, K), "bad shape"),
        ((codes.to(torch.int64), scales, N, K), "int32"),       # wrong element type
        ((codes, scales.float(), N, K), "int32"),
        ((torch.zeros(2 * cw, dtype=torch.int32)[::2], scales, N, K), "contiguous"),  # a strided view
    ]:
        with pytest.raises(binding.Itq3sError, match=what):
            binding._need_packed(*bad_args)
    with pytest.raises(binding.Itq3sError, match="status_flags"):
        binding._need_flags(torch.zeros(0, dtype=torch.int32))
    with pytest.raises(binding.Itq3sError, match="status_flags"):
        binding._need_flags(torch.zeros(1, dtype=torch.float32))
    binding._need_flags(None)
    binding._need_flags(torch.zeros(1, dtype=torch.int32))
