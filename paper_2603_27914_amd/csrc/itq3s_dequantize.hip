// Weight-side reconstruction (Alg. 2, Prop. 1): w_hat = H( d (q - z) ).
//
// q takes small integer values, so the transform of the digits is exact in any arithmetic that holds
// integers up to 512; the zero-point only reaches element 0 (H applied to a constant vector is a
// spike: H 1 = 16 e_0) and is folded in after the transform.  One rounding per output element.
//
// The 256-point transform runs on the matrix cores.  With the block written as a 16 x 16 matrix
// V[a][b] = v[16a + b], the Sylvester construction gives H_256 = H_16 (x) H_16, so
// (H_u v)[16a' + b'] = (H_16 V H_16)[a'][b'] with the +-1 matrix H_16.  The kernel forms the
// transpose, U^T = H_16 (V^T H_16): two 16x16x16 products on fp16 inputs (digits, then integers up
// to 32: all exact) with fp32 sums.  The accumulator layout of the first product is the B-operand
// layout of the second, and the transposed result leaves every lane with four consecutive output
// elements, e = 16 (l%16) + 4 (l/16) + 0..3: a wavefront stores one contiguous row segment.
// One wavefront per block; a workgroup of four wavefronts covers one 16-row tile, four rows each.
#include "itq3s_dev.h"
#include "itq3s_kernels.h"

namespace itq3s {

// (at least two wavefronts per SIMD: with a register budget of 256 the matrix instructions write ordinary
// vector registers; with the full 512 the compiler parks their results in accumulator registers and copies
// every one of them out)
// kSub: the sub-block-scale variant (Sec. 4.1: 116 bytes per block), w_hat = H( d (s_j q - z) ).  A lane's
// four digits belong to sub-blocks 2g (the first two) and 2g+1, whose scales are the two halves of
// the lane's own word of the sub-scale array; s q is exact in fp16, the first product (16 terms of one
// sub-block: a 16-bit number) is carried in two fp16 parts, the second adds 16 such terms in fp32.
template <bool kOutF16, bool kSub>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void dequantize_kernel(const uint32_t* __restrict__ codes, const uint32_t* __restrict__ scales,
                                                         const uint32_t* __restrict__ subscales, int64_t N, int KB, void* __restrict__ out, int64_t ldo,
                                                         uint32_t* __restrict__ flags) {
    const int tile = (int)blockIdx.x;
    const int nt = tile / KB, b = tile - nt * KB;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int r16 = lane & 15, g = lane >> 4;
    const uint32_t* t = codes + (int64_t)tile * kTileWords;

    half4 h;  // H_16[4g + j][r16]: B operand of the first product, A operand of the second
#pragma unroll
    for (int j = 0; j < 4; ++j) h[j] = (__builtin_popcount((4 * g + j) & r16) & 1) ? (_Float16)(-1.0f) : (_Float16)1.0f;

    // the four rows of this wavefront: loads first, arithmetic after
    u32x4 lo[4];
    u32x2 hi[4];
    uint32_t sw[4];
    uint32_t ssw[4];
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const int r = wave * 4 + rr;
        ssw[rr] = kSub ? subscales[(int64_t)tile * 64 + 16 * g + r] : 0u;
        // elements e = 64 g + 16 j + r16 (j = 0..3) sit in slot r16 of low-plane word j of storage lane
        // 16 g + r; their high bits in bit 16 (j & 1) + r16 of high-plane word j >> 1
        lo[rr] = *reinterpret_cast<const u32x4*>(t + 4 * (16 * g + r));
        hi[rr] = *reinterpret_cast<const u32x2*>(t + kTileLoWords + 2 * (16 * g + r));
        sw[rr] = scales[(int64_t)tile * kTileRows + r];
    }
    uint32_t bad = 0;
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const int r = wave * 4 + rr;
        const int64_t n = (int64_t)nt * kTileRows + r;  // (rows past N exist in storage; only their store is skipped)
        // The lane's four codes sit in slot r16 of the four low-plane words.  Two at a time they are
        // OR-ed into the mantissa of the half 1024.0, whose lowest mantissa bit weighs exactly 1:
        // 1024 + c, minus 1025, is the digit c - 1 (exact).  A code 3, or any high-plane bit of the
        // row (every lane of the row group reads the same words), is a format error.
        const uint32_t sh = 2u * (uint32_t)r16;
        const uint32_t c0 = (lo[rr].x >> sh) & 3u, c1 = (lo[rr].y >> sh) & 3u, c2 = (lo[rr].z >> sh) & 3u, c3 = (lo[rr].w >> sh) & 3u;
        uint32_t p01 = c0 | (c1 << 16), p23 = c2 | (c3 << 16);
        bad |= (((p01 & (p01 >> 1)) | (p23 & (p23 >> 1))) & 0x00010001u) | hi[rr].x | hi[rr].y;
        if (__builtin_amdgcn_ballot_w64((hi[rr].x | hi[rr].y) != 0u) != 0ull) {
            // (malformed input only) the high bits count 4: the digit is still code - 1
            p01 |= (((hi[rr].x >> r16) & 1u) << 2) | (((hi[rr].x >> (16 + r16)) & 1u) << 18);
            p23 |= (((hi[rr].y >> r16) & 1u) << 2) | (((hi[rr].y >> (16 + r16)) & 1u) << 18);
        }
        const half2v bias = {(_Float16)(-1025.0f), (_Float16)(-1025.0f)};
        const half2v v01 = __builtin_bit_cast(half2v, p01 | 0x64006400u) + bias, v23 = __builtin_bit_cast(half2v, p23 | 0x64006400u) + bias;
        half4 v = {v01[0], v01[1], v23[0], v23[1]};
        if constexpr (kSub) {
            const _Float16 s_lo = __builtin_bit_cast(_Float16, (uint16_t)(ssw[rr] & 0xffffu)), s_hi = __builtin_bit_cast(_Float16, (uint16_t)(ssw[rr] >> 16));
            v = half4{v[0] * s_lo, v[1] * s_lo, v[2] * s_hi, v[3] * s_hi};
        }
        const floatx4 zero = {0.f, 0.f, 0.f, 0.f};
        const floatx4 T = __builtin_amdgcn_mfma_f32_16x16x16f16(v, h, zero, 0, 0, 0);  // V^T H_16, |.| <= 16 * 6
        const half4 th = {(_Float16)T[0], (_Float16)T[1], (_Float16)T[2], (_Float16)T[3]};
        floatx4 U = __builtin_amdgcn_mfma_f32_16x16x16f16(h, th, zero, 0, 0, 0);
        if constexpr (kSub) {
            const half4 tl = {(_Float16)(T[0] - (float)th[0]), (_Float16)(T[1] - (float)th[1]), (_Float16)(T[2] - (float)th[2]), (_Float16)(T[3] - (float)th[3])};
            U = __builtin_amdgcn_mfma_f32_16x16x16f16(h, tl, U, 0, 0, 0);
        }
        const float d16 = f16_bits_to_f32(sw[rr] & 0xffffu) * 0.0625f;  // d / 16: exact, so one rounding per output as before
        const float z = f16_bits_to_f32(sw[rr] >> 16);
        float f[4] = {U[0], U[1], U[2], U[3]};
        if (lane == 0) f[0] = f[0] - 256.0f * z;  // H_u applied to the constant -z
#pragma unroll
        for (int i = 0; i < 4; ++i) f[i] = d16 * f[i];
        const int64_t off = n * ldo + (int64_t)b * kBlock + 16 * r16 + 4 * g;
        if (n < N) {
            if (kOutF16) {
                half4 o = {(_Float16)f[0], (_Float16)f[1], (_Float16)f[2], (_Float16)f[3]};
                *reinterpret_cast<half4*>(reinterpret_cast<_Float16*>(out) + off) = o;
            } else {
                *reinterpret_cast<float4*>(reinterpret_cast<float*>(out) + off) = make_float4(f[0], f[1], f[2], f[3]);
            }
        }
    }
    if (flags != nullptr && __builtin_amdgcn_ballot_w64(bad != 0u) != 0ull && lane == 0) atomicOr(flags, kFlagBadCode);
}

int launch_dequantize(const uint32_t* codes, const uint32_t* scales, const uint32_t* subscales, int64_t N, int64_t K, void* out, int out_f16,
                      int64_t ldo, uint32_t* flags, hipStream_t stream) {
    const int64_t tiles = ((N + 15) / 16) * (K / kBlock);
    const int KB = (int)(K / kBlock);
    const dim3 grid((unsigned)tiles), block(256);
    if (subscales != nullptr) {
        if (out_f16) hipLaunchKernelGGL((dequantize_kernel<true, true>), grid, block, 0, stream, codes, scales, subscales, N, KB, out, ldo, flags);
        else hipLaunchKernelGGL((dequantize_kernel<false, true>), grid, block, 0, stream, codes, scales, subscales, N, KB, out, ldo, flags);
    } else {
        if (out_f16) hipLaunchKernelGGL((dequantize_kernel<true, false>), grid, block, 0, stream, codes, scales, subscales, N, KB, out, ldo, flags);
        else hipLaunchKernelGGL((dequantize_kernel<false, false>), grid, block, 0, stream, codes, scales, subscales, N, KB, out, ldo, flags);
    }
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

}  // namespace itq3s
