"""Pins for the oracle's sub-block-scale variant (Sec. 4.1: 8 fp16 sub-scales, 116 bytes per block).

The paper names the option and its byte budget and nothing else, so what is pinned here is (i) that
budget, (ii) that the variant IS the base format when every sub-scale is 1, (iii) the reading written
in the oracle's header, against a dense long-double implementation that shares nothing with the
oracle's butterflies or sums, (iv) Prop. 1 with the scaled digit against a dense Hadamard matrix,
(v) the isometry identity and the behaviour the option exists for (it helps where sub-block energies
differ and cannot hurt much where they do not).  Everything beyond is "parity unpinned"."""
import numpy as np
import pytest

from paper_2603_27914_amd import synth
from tests.packed_inputs import unpack_numpy
from tests.test_oracle_pins import dense_hu, np_f16


def unpack_subs(subs, N, K):
    """Second reading of the sub-scale storage, from its description: -> s float64 [N, KB, 8]."""
    KB, NT = K // 256, (N + 15) // 16
    t = subs.reshape(NT, KB, 4, 16)  # [tile row][block][quarter g][row r]
    lo = (t & 0xFFFF).astype(np.uint16).view(np.float16).astype(np.float64)
    hi = (t >> 16).astype(np.uint16).view(np.float16).astype(np.float64)
    s = np.stack([lo, hi], axis=3)  # [NT][KB][g][2][r] -> sub-block 2g + h
    s = s.transpose(0, 4, 1, 2, 3).reshape(NT * 16, KB, 8)
    return s[:N]


def test_byte_budget(ref):
    N, K = 40, 768
    assert ref.codes_words(N, K) * 4 + ref.scales_words(N, K) * 4 + ref.subscales_words(N, K) * 4 == 3 * 3 * 16 * 116
    assert (96 + 2 + 2 + 16) * 8 / 256 == 3.625


def independent_sub(w):
    H = dense_hu().astype(np.longdouble)
    wt = (H @ w.astype(np.longdouble)) / np.longdouble(16)
    mu = wt.mean()
    sigma = np.sqrt(((wt - mu) ** 2).mean())
    d = float(np.float16(np.float32(0.7979 * float(sigma))))
    z = -np.floor(float(mu) / d + 0.5)
    s = np.empty(8)
    for j in range(8):
        sj = np.sqrt(((wt[32 * j : 32 * j + 32] - mu) ** 2).mean())
        s[j] = float(np.float16(np.float32(0.7979 * float(sj) / d)))
    return wt, d, z, s


@pytest.mark.parametrize("seed", range(6))
def test_block_against_dense_definition(ref, seed):
    rng = np.random.default_rng(500 + seed)
    w = (0.02 * rng.standard_t(4.0, size=256)).astype(np.float32)
    if seed % 2:
        w[0] = np.float32(0.9)  # non-zero zero-point
    if seed >= 3:
        # make the energy of the rotated sub-blocks differ: add a multiple of a few Hadamard rows
        H = dense_hu().astype(np.float64) / 16.0
        boost = np.zeros(256)
        boost[40:60] = rng.normal(size=20) * 0.3
        w = (w + H @ boost).astype(np.float32)
    codes, word, sbits, flags = ref.quantize_block_sub(w)
    assert flags == 0
    wt, d, z, s = independent_sub(w)
    assert np_f16(word) == d and np_f16(word >> 16) == z
    got_s = sbits.view(np.float16).astype(np.float64)
    assert np.array_equal(got_s, s)
    if seed >= 3:
        assert got_s[1] > 2.0 * np.median(got_s)
    x = (wt / np.longdouble(d) + np.longdouble(z)) / np.repeat(s, 32).astype(np.longdouble) + np.longdouble(0.5)
    q = np.clip(np.floor(x), -1, 1).astype(np.int64)
    safe = np.abs(x - np.round(x)) > 1e-9
    assert safe.sum() >= 250
    assert np.array_equal(codes.astype(np.int64)[safe] - 1, q[safe])
    # base fields are those of the base format
    c0, word0, _ = ref.quantize_block(w)
    assert word0 == word


def test_unit_sub_scales_are_the_base_format(ref):
    N, K = 24, 512
    W = synth.weights(N, K, "sub-unit")
    W[:, 0] += 0.5
    codes, scales, _ = ref.quantize(W)
    ones = np.full(ref.subscales_words(N, K), 0x3C003C00, dtype=np.uint32)
    assert np.array_equal(ref.dequantize_sub(codes, scales, ones, N, K), ref.dequantize(codes, scales, N, K))
    X = synth.activations(3, K, "sub-unit")
    assert np.array_equal(ref.matmul_sub(codes, scales, ones, N, K, X), ref.matmul(codes, scales, N, K, X))


def test_packed_layout_and_dequantize_against_dense(ref):
    N, K = 40, 768
    W = synth.weights(N, K, "sub-deq")
    W[:, 0] += 0.4
    codes, scales, subs, flags = ref.quantize_sub(W)
    assert flags == 0
    c, d, z = unpack_numpy(codes, scales, N, K)
    s = unpack_subs(subs, N, K)
    for n in (0, 15, 16, 39):
        for b in range(3):
            cb, word, sb, _ = ref.quantize_block_sub(W[n, 256 * b : 256 * b + 256])
            assert np.array_equal(c[n, 256 * b : 256 * b + 256], cb)
            assert np.array_equal(s[n, b], sb.view(np.float16).astype(np.float64))
            assert d[n, b] == np_f16(word)
    spad = unpack_subs(subs, 48, K)
    assert not spad[40:].any()
    H = dense_hu().astype(np.float64) / 16.0
    want = np.empty((N, K))
    for b in range(K // 256):
        v = d[:, b : b + 1] * (np.repeat(s[:, b, :], 32, axis=1) * (c[:, 256 * b : 256 * b + 256] - 1) - z[:, b : b + 1])
        want[:, 256 * b : 256 * b + 256] = v @ H.T
    got = ref.dequantize_sub(codes, scales, subs, N, K)
    assert np.allclose(got, want, rtol=0, atol=1e-14 * np.abs(want).max() * 256)
    # isometry: the reconstruction error equals the coding error in the rotated domain
    for n in (3, 27):
        wt = ref.forward_block(W[n, :256])
        v = d[n, 0] * (np.repeat(s[n, 0], 32) * (c[n, :256] - 1) - z[n, 0])
        assert abs(np.linalg.norm(got[n, :256] - W[n, :256].astype(np.float64)) - np.linalg.norm(v - wt)) <= 1e-12 * np.linalg.norm(wt) + 1e-9 * np.linalg.norm(v - wt)


def test_matmul_sub_brute_force(ref):
    N, K, M = 5, 512, 3
    W = synth.weights(N, K, "sub-mm")
    codes, scales, subs, _ = ref.quantize_sub(W)
    What = ref.dequantize_sub(codes, scales, subs, N, K)
    X = synth.activations(M, K, "sub-mm")
    want = np.array([[sum(float(X[m, k]) * What[n, k] for k in range(K)) for n in range(N)] for m in range(M)])
    got = ref.matmul_sub(codes, scales, subs, N, K, X)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-14)


def test_sub_scales_help_where_sub_block_energies_differ(ref):
    """What the option is for: rotated blocks whose 32-coefficient sub-blocks differ in energy get a
    finer grid where they are quiet.  On i.i.d. weights the rotation has already equalised the
    energies and the gain is small, but the variant is never much worse."""
    rng = np.random.default_rng(9)
    H = dense_hu().astype(np.float64) / 16.0
    gains = []
    for trial in range(40):
        prof = np.repeat(np.exp(rng.normal(size=8)), 32)           # per-sub-block standard deviation
        wt = rng.normal(size=256) * prof * 0.02
        w = (H @ wt).astype(np.float32)                             # H is its own inverse
        c0, word0, _ = ref.quantize_block(w)
        c1, word1, sb, _ = ref.quantize_block_sub(w)
        d = np_f16(word0)
        z = np_f16(word0 >> 16)
        s = np.repeat(sb.view(np.float16).astype(np.float64), 32)
        wt64 = ref.forward_block(w)
        e0 = np.linalg.norm(d * ((c0.astype(np.float64) - 1) - z) - wt64)
        e1 = np.linalg.norm(d * (s * (c1.astype(np.float64) - 1) - z) - wt64)
        gains.append(e1 / e0)
    assert np.median(gains) < 0.9
    iid = []
    for trial in range(40):
        w = (0.02 * rng.standard_t(4.0, size=256)).astype(np.float32)
        c0, word0, _ = ref.quantize_block(w)
        c1, word1, sb, _ = ref.quantize_block_sub(w)
        d, z = np_f16(word0), np_f16(word0 >> 16)
        s = np.repeat(sb.view(np.float16).astype(np.float64), 32)
        wt64 = ref.forward_block(w)
        iid.append(np.linalg.norm(d * (s * (c1.astype(np.float64) - 1) - z) - wt64) / np.linalg.norm(d * ((c0.astype(np.float64) - 1) - z) - wt64))
    assert np.median(iid) < 1.02 and max(iid) < 1.15


def test_degenerate_and_nonfinite_blocks(ref):
    codes, word, sb, flags = ref.quantize_block_sub(np.zeros(256, dtype=np.float32))
    assert word == 0 and not sb.any() and np.all(codes == 1) and flags == 0
    w = np.zeros(256, dtype=np.float32)
    w[7] = np.inf
    codes, word, sb, flags = ref.quantize_block_sub(w)
    assert word == 0 and not sb.any() and np.all(codes == 1) and flags & ref.FLAG_NONFINITE
    # one quiet sub-block in the rotated domain gets a sub-scale far below the others
    H = dense_hu().astype(np.float64) / 16.0
    wt = np.random.default_rng(2).normal(size=256) * 0.05
    wt[64:96] = wt.mean()  # sub-block 2 sits (almost) on the mean
    w = (H @ wt).astype(np.float32)
    codes, word, sb, flags = ref.quantize_block_sub(w)
    s = sb.view(np.float16).astype(np.float64)
    assert s[2] < 0.05 * np.median(s)
