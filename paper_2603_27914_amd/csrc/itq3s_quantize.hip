// Offline quantizer (Alg. 1, Def. 1): one wavefront per 256-element block, fp64 arithmetic in a
// fixed order so that the packed output is bit-identical on any IEEE-754 machine.
//
// Lane l holds elements 4l..4l+3.  Butterfly stages with distance 1 and 2 stay inside the lane,
// distances 4..128 exchange with lane l^1 .. l^32.  This file must be compiled with floating
// point contraction off: every add, subtract and multiply below rounds on its own.
#include "itq3s_dev.h"
#include "itq3s_kernels.h"

namespace itq3s {

constexpr double kTStar = 0.7979;  // optimal ternary scale / sigma (Sec. 3.3, App. A)

// Sum over the 256 elements of a block, pairwise: neighbours first, then distance 2, 4, ... 128.
// Addition is commutative bit for bit, so every lane ends with the same value.
__device__ __forceinline__ double block_pairwise_sum(double v0, double v1, double v2, double v3) {
    double t = (v0 + v1) + (v2 + v3);
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) t = t + xor_lane_f64(t, m);
    return t;
}

__global__ __launch_bounds__(256) void quantize_kernel(const float* __restrict__ W, int64_t N, int64_t K, int64_t ldw,
                                                       uint32_t* __restrict__ codes, uint32_t* __restrict__ scales,
                                                       uint32_t* __restrict__ flags) {
    __shared__ uint32_t tile_lds[kTileWords];
    __shared__ uint32_t scale_lds[kTileRows];

    const int64_t KB = K / kBlock;
    const int64_t tile = blockIdx.x;  // nt * KB + b
    const int64_t nt = tile / KB, b = tile - nt * KB;
    const int lane = lane_id(), wave = threadIdx.x >> 6;

    if (threadIdx.x < kTileWords - kTileLoWords) tile_lds[kTileLoWords + threadIdx.x] = 0u;  // high plane: always 0
    uint32_t my_flags = 0;

    for (int rr = 0; rr < 4; ++rr) {
        const int r = wave * 4 + rr;
        const int64_t n = nt * kTileRows + r;
        uint32_t code_byte = 0x55u;  // four codes "1" = digit 0
        uint32_t word = 0u;
        if (n < N) {
            const float4 w4 = *reinterpret_cast<const float4*>(W + n * ldw + b * kBlock + 4 * lane);
            double a0 = (double)w4.x, a1 = (double)w4.y, a2 = (double)w4.z, a3 = (double)w4.w;
            const bool finite = isfinite(w4.x) && isfinite(w4.y) && isfinite(w4.z) && isfinite(w4.w);
            if (__builtin_amdgcn_ballot_w64(!finite) != 0ull) {
                my_flags |= kFlagNonFinite;
            } else {
                // w' = H w: stages 1, 2 in registers ...
                double t0 = a0 + a1, t1 = a0 - a1, t2 = a2 + a3, t3 = a2 - a3;
                a0 = t0 + t2; a2 = t0 - t2; a1 = t1 + t3; a3 = t1 - t3;
                // ... stages 4 .. 128 across lanes: the lower index gets u+v, the higher one u-v
#pragma unroll
                for (int m = 1; m < 64; m <<= 1) {
                    const bool upper = (lane & m) != 0;
                    const double p0 = xor_lane_f64(a0, m), p1 = xor_lane_f64(a1, m);
                    const double p2 = xor_lane_f64(a2, m), p3 = xor_lane_f64(a3, m);
                    a0 = upper ? (p0 - a0) : (a0 + p0);
                    a1 = upper ? (p1 - a1) : (a1 + p1);
                    a2 = upper ? (p2 - a2) : (a2 + p2);
                    a3 = upper ? (p3 - a3) : (a3 + p3);
                }
                a0 = a0 * 0.0625; a1 = a1 * 0.0625; a2 = a2 * 0.0625; a3 = a3 * 0.0625;

                const double mu = block_pairwise_sum(a0, a1, a2, a3) / 256.0;
                const double e0 = a0 - mu, e1 = a1 - mu, e2 = a2 - mu, e3 = a3 - mu;
                const double sigma = sqrt(block_pairwise_sum(e0 * e0, e1 * e1, e2 * e2, e3 * e3) / 256.0);
                double d64 = kTStar * sigma;
                if (d64 > 65504.0) { d64 = 65504.0; my_flags |= kFlagScaleSat; }
                const _Float16 dh = (_Float16)(float)d64;  // two roundings to nearest even, as specified
                const double d = (double)dh;
                if (d > 0.0) {
                    const double rnd = floor(mu / d + 0.5);
                    double z = 0.0 - rnd;
                    if (z > 2048.0) { z = 2048.0; my_flags |= kFlagZClamp; }
                    if (z < -2048.0) { z = -2048.0; my_flags |= kFlagZClamp; }
                    const double t_hi = (0.5 - z) * d, t_lo = (-0.5 - z) * d;  // exact products
                    const uint32_t c0 = a0 >= t_hi ? 2u : (a0 < t_lo ? 0u : 1u);
                    const uint32_t c1 = a1 >= t_hi ? 2u : (a1 < t_lo ? 0u : 1u);
                    const uint32_t c2 = a2 >= t_hi ? 2u : (a2 < t_lo ? 0u : 1u);
                    const uint32_t c3 = a3 >= t_hi ? 2u : (a3 < t_lo ? 0u : 1u);
                    code_byte = c0 | (c1 << 2) | (c2 << 4) | (c3 << 6);
                    const _Float16 zh = (_Float16)(float)z;
                    word = (uint32_t)__builtin_bit_cast(uint16_t, dh) | ((uint32_t)__builtin_bit_cast(uint16_t, zh) << 16);
                }
            }
        }
        // elements 4l..4l+3 of row r: low-plane word 4*(16*(l>>4) + r) + ((l>>2)&3), byte l&3
        const int word_idx = 4 * (16 * (lane >> 4) + r) + ((lane >> 2) & 3);
        reinterpret_cast<unsigned char*>(tile_lds)[4 * word_idx + (lane & 3)] = (unsigned char)code_byte;
        if (lane == 0) scale_lds[r] = word;
    }
    __syncthreads();
    uint32_t* out = codes + tile * kTileWords;
    out[threadIdx.x] = tile_lds[threadIdx.x];
    if (threadIdx.x < kTileWords - 256) out[256 + threadIdx.x] = tile_lds[256 + threadIdx.x];
    if (threadIdx.x < kTileRows) scales[tile * kTileRows + threadIdx.x] = scale_lds[threadIdx.x];
    if (flags != nullptr && my_flags != 0u && lane == 0) atomicOr(flags, my_flags);
}

int launch_quantize(const float* W, int64_t N, int64_t K, int64_t ldw, uint32_t* codes, uint32_t* scales, uint32_t* flags,
                    hipStream_t stream) {
    const int64_t tiles = ((N + 15) / 16) * (K / kBlock);
    hipLaunchKernelGGL(quantize_kernel, dim3((unsigned)tiles), dim3(256), 0, stream, W, N, K, ldw, codes, scales, flags);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

}  // namespace itq3s
