// Offline quantizer (Alg. 1, Def. 1) in fp64, every operation in a fixed order so that the packed
// output is bit-identical on any IEEE-754 machine.
//
// A block (256 consecutive channels of one row) is held by 16 lanes, 16 consecutive elements each:
// a wavefront works on four rows of a storage tile at once, a workgroup of four wavefronts on the
// whole 16-row tile.  Butterfly stages with distance 1, 2, 4, 8 stay inside the lane; distances
// 16 .. 128 exchange with lane l^1, l^2, l^4, l^8 of the same row of 16 lanes through the LDS
// crossbar (swizzles: no memory access).  The 16 codes of a lane are exactly one low-plane
// word of the packed tile, so the result is stored straight from registers.  This file must be
// compiled with floating point contraction off: every add, subtract and multiply below rounds on
// its own.
#include "itq3s_dev.h"
#include "itq3s_kernels.h"

namespace itq3s {

constexpr double kTStar = 0.7979;  // optimal ternary scale / sigma (Sec. 3.3, App. A)

// One cross-lane butterfly stage: the lower lane of a pair gets u + v, the upper one u - v (u the
// lower lane's value).  Both are one fused multiply-add (+-1) * own + other: the product is exact,
// so the upper lane's (-v) + u is u - v bit for bit.
template <int MASK>
__device__ __forceinline__ void cross_stage(double (&a)[16], int l16) {
    const double sign = (l16 & MASK) ? -1.0 : 1.0;
#pragma unroll
    for (int i = 0; i < 16; ++i) a[i] = __builtin_fma(a[i], sign, row_xor_f64<MASK>(a[i]));  // (+-a) + p, one rounding
}

// Sum over the 256 elements of a block, pairwise: neighbours first, then distance 2, 4, ... 128.
// Addition is commutative bit for bit, so every lane of the row ends with the same value.
__device__ __forceinline__ double block_pairwise_sum(const double (&v)[16]) {
    double t[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) t[i] = v[2 * i] + v[2 * i + 1];
#pragma unroll
    for (int i = 0; i < 4; ++i) t[i] = t[2 * i] + t[2 * i + 1];
    t[0] = t[0] + t[1];
    t[1] = t[2] + t[3];
    double s = t[0] + t[1];
    s = s + row_xor_f64<1>(s);
    s = s + row_xor_f64<2>(s);
    s = s + row_xor_f64<4>(s);
    s = s + row_xor_f64<8>(s);
    return s;
}

__global__ __launch_bounds__(256) void quantize_kernel(const float* __restrict__ W, int64_t N, int64_t K, int64_t ldw,
                                                       uint32_t* __restrict__ codes, uint32_t* __restrict__ scales,
                                                       uint32_t* __restrict__ flags, int KB) {
    const int tile = (int)blockIdx.x;  // nt * KB + b
    const int nt = tile / KB, b = tile - nt * KB;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int l16 = lane & 15, r = 4 * wave + (lane >> 4);
    const int64_t n = (int64_t)nt * kTileRows + r;
    uint32_t* const out = codes + (int64_t)tile * kTileWords;

    // high plane: always 0 on encode (128 words, threads 0..127)
    if (threadIdx.x < kTileWords - kTileLoWords) out[kTileLoWords + threadIdx.x] = 0u;

    uint32_t my_flags = 0;
    uint32_t lo_word = 0x55555555u;  // sixteen codes "1" = digit 0
    uint32_t scale_word = 0u;
    if (n < N) {  // (uniform over the 16 lanes of a row; the moves below never leave the row)
        const float4* src = reinterpret_cast<const float4*>(W + n * ldw + (int64_t)b * kBlock + 16 * l16);
        const float4 w0 = src[0], w1 = src[1], w2 = src[2], w3 = src[3];
        const float wf[16] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w, w2.x, w2.y, w2.z, w2.w, w3.x, w3.y, w3.z, w3.w};
        bool finite = true;
        double a[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            finite = finite && isfinite(wf[i]);
            a[i] = (double)wf[i];
        }
        // any non-finite weight among the 16 lanes of this row?
        const unsigned long long bal = __builtin_amdgcn_ballot_w64(!finite);
        const bool row_bad = ((bal >> (lane & 48)) & 0xffffull) != 0ull;

        // w' = H w: stages 1, 2, 4, 8 in registers (the lower index gets u+v, the higher one u-v) ...
#pragma unroll
        for (int s = 1; s < 16; s <<= 1)
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if ((i & s) == 0) {
                    const double u = a[i], v = a[i + s];
                    a[i] = u + v;
                    a[i + s] = u - v;
                }
        // ... stages 16 .. 128 across the lanes of the row
        cross_stage<1>(a, l16);
        cross_stage<2>(a, l16);
        cross_stage<4>(a, l16);
        cross_stage<8>(a, l16);
#pragma unroll
        for (int i = 0; i < 16; ++i) a[i] = a[i] * 0.0625;

        const double mu = block_pairwise_sum(a) / 256.0;
        double e2[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const double e = a[i] - mu;
            e2[i] = e * e;
        }
        const double sigma = sqrt(block_pairwise_sum(e2) / 256.0);
        double d64 = kTStar * sigma;
        bool sat = false, zclamp = false;
        if (d64 > 65504.0) { d64 = 65504.0; sat = true; }
        const _Float16 dh = (_Float16)(float)d64;  // two roundings to nearest even, as specified
        const double d = (double)dh;
        const bool live = !row_bad && d > 0.0;  // otherwise the block is stored as zeros
        const double rnd = floor(mu / (live ? d : 1.0) + 0.5);
        double z = 0.0 - rnd;
        if (z > 2048.0) { z = 2048.0; zclamp = true; }
        if (z < -2048.0) { z = -2048.0; zclamp = true; }
        const double t_hi = (0.5 - z) * d, t_lo = (-0.5 - z) * d;  // exact products
        uint32_t word = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const uint32_t c = a[i] >= t_hi ? 2u : (a[i] < t_lo ? 0u : 1u);
            word |= c << (2 * i);
        }
        if (live) {
            lo_word = word;
            const _Float16 zh = (_Float16)(float)z;
            scale_word = (uint32_t)__builtin_bit_cast(uint16_t, dh) | ((uint32_t)__builtin_bit_cast(uint16_t, zh) << 16);
            if (zclamp) my_flags |= kFlagZClamp;
        }
        if (row_bad) my_flags |= kFlagNonFinite;
        else if (sat) my_flags |= kFlagScaleSat;
    }
    // elements 16 l16 .. 16 l16 + 15 of row r: low-plane word 4*(16*(l16>>2) + r) + (l16&3)
    out[4 * (16 * (l16 >> 2) + r) + (l16 & 3)] = lo_word;
    if (l16 == 0) scales[(int64_t)tile * kTileRows + r] = scale_word;
    if (flags != nullptr && __builtin_amdgcn_ballot_w64(my_flags != 0u) != 0ull) {
        // one atomic per wavefront: OR of the flags of its lanes
        uint32_t f = my_flags;
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) f |= (uint32_t)__shfl_xor((int)f, m, 64);
        if (lane == 0) atomicOr(flags, f);
    }
}

int launch_quantize(const float* W, int64_t N, int64_t K, int64_t ldw, uint32_t* codes, uint32_t* scales, uint32_t* flags,
                    hipStream_t stream) {
    const int64_t tiles = ((N + 15) / 16) * (K / kBlock);
    hipLaunchKernelGGL(quantize_kernel, dim3((unsigned)tiles), dim3(256), 0, stream, W, N, K, ldw, codes, scales, flags, (int)(K / kBlock));
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

}  // namespace itq3s
