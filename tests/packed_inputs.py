"""Random packed tensors for tests that are too large to run a quantizer first.

Test input generation only: the bytes written here go to the HIP path and to the CPU oracle alike,
which both decode them by their own reading of the format (include/itq3s.h), so a mistake in this
writer shows up as two decoders agreeing on a different tensor, not as a false pass."""
import numpy as np

from paper_2603_27914_amd import synth


def random_packed(N, K, *key, z_fraction=0.001):
    """Random valid packed tensor: codes uniform in {0,1,2}, fp16 scales near 0.016, a fraction of
    the blocks with a non-zero integer zero-point.  Rows >= N of the last 16-row tile hold code 1
    and scale word 0, as the format requires.  Returns (codes uint32, scales uint32) in the tiled
    layout: 16-row tiles of 384 words (256 low-plane words of sixteen 2-bit fields, 128 high-plane
    words, all zero)."""
    g = synth._rng("P", N, K, *key)
    NT, KB = (N + 15) // 16, K // 256
    # [tile][lane = 16 * quarter + row][word of the lane][field]
    c = g.integers(0, 3, size=(NT * KB, 64, 4, 16), dtype=np.uint32)
    d = (0.016 * np.exp(0.25 * g.standard_normal(size=(NT * KB, 16)))).astype(np.float16)
    z = np.zeros((NT * KB, 16), dtype=np.float16)
    nz = g.random((NT * KB, 16)) < z_fraction
    z[nz] = g.integers(-3, 4, size=int(nz.sum())).astype(np.float16)
    pad = NT * 16 - N
    if pad:
        last = np.arange(NT * KB).reshape(NT, KB)[-1]  # the tiles of the last row tile
        rows = np.arange(64) % 16 >= 16 - pad          # lanes that belong to rows >= N
        c[np.ix_(last, np.nonzero(rows)[0])] = 1
        d[last, 16 - pad :] = 0
        z[last, 16 - pad :] = 0
    lo = np.zeros((NT * KB, 64, 4), dtype=np.uint32)
    for s in range(16):
        lo |= c[..., s] << np.uint32(2 * s)
    codes = np.zeros((NT * KB, 384), dtype=np.uint32)
    codes[:, :256] = lo.reshape(NT * KB, 256)
    scales = d.view(np.uint16).astype(np.uint32) | (z.view(np.uint16).astype(np.uint32) << np.uint32(16))
    return codes.reshape(-1), scales.reshape(-1)


def unpack_numpy(codes, scales, N, K):
    """Second implementation of the storage layout, written from its description alone.
    -> (c int64 [N,K], d float64 [N,KB], z float64 [N,KB])."""
    KB, NT = K // 256, (N + 15) // 16
    t = codes.reshape(NT, KB, 384)
    e = np.arange(256)
    lane_g, i = e >> 6, e & 63
    c = np.zeros((NT * 16, K), dtype=np.int64)
    for r in range(16):
        lane = 16 * lane_g + r
        lo = (t[:, :, 4 * lane + (i >> 4)] >> (2 * (i & 15)).astype(np.uint32)) & 3
        hi = (t[:, :, 256 + 2 * lane + (i >> 5)] >> (i & 31).astype(np.uint32)) & 1
        c[r::16, :] = (lo | (hi << 2)).reshape(NT, K)
    s = scales.reshape(NT, KB, 16).transpose(0, 2, 1).reshape(NT * 16, KB)
    d = (s & 0xFFFF).astype(np.uint16).view(np.float16).astype(np.float64)
    z = (s >> 16).astype(np.uint16).view(np.float16).astype(np.float64)
    return c[:N], d[:N], z[:N]
