// Weight-side reconstruction (Alg. 2, Prop. 1): w_hat = H( d (q - z) ).
//
// q - z takes small integer values, so the eight butterfly stages run in int32 and are exact; the
// zero-point only reaches element 0 (H applied to a constant vector is a spike: H 1 = 16 e_0) and
// is folded in after the transform.  One rounding per output element.  One wavefront per block,
// lane l holds elements 4l..4l+3; a workgroup of four wavefronts covers one 16-row tile.
#include "itq3s_dev.h"
#include "itq3s_kernels.h"

namespace itq3s {

template <bool kOutF16>
__global__ __launch_bounds__(256) void dequantize_kernel(const uint32_t* __restrict__ codes, const uint32_t* __restrict__ scales,
                                                         int64_t N, int64_t K, void* __restrict__ out, int64_t ldo,
                                                         uint32_t* __restrict__ flags) {
    const int64_t KB = K / kBlock;
    const int64_t tile = blockIdx.x;
    const int64_t nt = tile / KB, b = tile - nt * KB;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const uint32_t* t = codes + tile * kTileWords;
    const int g = lane >> 4, w = (lane >> 2) & 3, q4 = lane & 3;
    bool bad = false;

    for (int rr = 0; rr < 4; ++rr) {
        const int r = wave * 4 + rr;
        const int64_t n = nt * kTileRows + r;
        if (n >= N) break;
        const uint32_t lo = t[4 * (16 * g + r) + w];
        const uint32_t hi = t[kTileLoWords + 2 * (16 * g + r) + (w >> 1)];
        const uint32_t sw = scales[tile * kTileRows + r];
        const uint32_t lo_byte = (lo >> (8 * q4)) & 0xffu;
        const uint32_t hi_nib = (hi >> (16 * (w & 1) + 4 * q4)) & 0xfu;
        int v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t c = ((lo_byte >> (2 * i)) & 3u) | (((hi_nib >> i) & 1u) << 2);
            bad |= c > 2u;
            v[i] = (int)c - 1;
        }
        // unnormalised Hadamard butterflies: distances 1, 2 in registers, 4..128 across lanes
        int t0 = v[0] + v[1], t1 = v[0] - v[1], t2 = v[2] + v[3], t3 = v[2] - v[3];
        v[0] = t0 + t2; v[2] = t0 - t2; v[1] = t1 + t3; v[3] = t1 - t3;
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) {
            const bool upper = (lane & m) != 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int p = xor_lane_i32(v[i], m);
                v[i] = upper ? (p - v[i]) : (v[i] + p);
            }
        }
        const float d = f16_bits_to_f32(sw & 0xffffu);
        const float z = f16_bits_to_f32(sw >> 16);
        float f[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) f[i] = (float)v[i];
        if (lane == 0) f[0] = f[0] - 256.0f * z;  // H_u applied to the constant -z
#pragma unroll
        for (int i = 0; i < 4; ++i) f[i] = (d * f[i]) * 0.0625f;
        const int64_t off = n * ldo + b * kBlock + 4 * lane;
        if (kOutF16) {
            half4 h = {(_Float16)f[0], (_Float16)f[1], (_Float16)f[2], (_Float16)f[3]};
            *reinterpret_cast<half4*>(reinterpret_cast<_Float16*>(out) + off) = h;
        } else {
            *reinterpret_cast<float4*>(reinterpret_cast<float*>(out) + off) = make_float4(f[0], f[1], f[2], f[3]);
        }
    }
    if (flags != nullptr && bad) atomicOr(flags, kFlagBadCode);
}

int launch_dequantize(const uint32_t* codes, const uint32_t* scales, int64_t N, int64_t K, void* out, int out_f16, int64_t ldo,
                      uint32_t* flags, hipStream_t stream) {
    const int64_t tiles = ((N + 15) / 16) * (K / kBlock);
    if (out_f16)
        hipLaunchKernelGGL(dequantize_kernel<true>, dim3((unsigned)tiles), dim3(256), 0, stream, codes, scales, N, K, out, ldo, flags);
    else
        hipLaunchKernelGGL(dequantize_kernel<false>, dim3((unsigned)tiles), dim3(256), 0, stream, codes, scales, N, K, out, ldo, flags);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

}  // namespace itq3s
