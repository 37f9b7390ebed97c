// Block-size ablation (Sec. 6, "Ablation: FWHT Block Size"): the rotate - quantize - reconstruct round
// trip with transform lengths n = 32 .. 512 instead of 256, without the packed format.
//
// Per block of n consecutive channels of a row:  w' = (H_u w) c_n,  d = 0.7979 sigma(w') -> fp16,
// z = -floor(mu/d + 1/2), codes by the exact thresholds (Alg. 1, Def. 1 as in the quantizer), then
// w_hat = (d (H_u (q - z))) c_n (Alg. 2, Prop. 1).  c_n is the fp64 value of 1/sqrt(n), one
// multiplication after the butterflies.  Everything up to the codes is fp64 in a fixed order
// (bit-identical to a serial evaluation); the reconstruction uses integer-valued fp64 butterflies
// (exact) and rounds once to fp32.
//
// A block is held by n/16 lanes, 16 consecutive elements each; a wavefront covers 1024 consecutive
// channels of a row (64/(n/16) blocks at once).  Stages 1..8 stay in the lane, the longer ones
// exchange with lane l^1, l^2, l^4, l^8 and, for n = 512, l^16 (swizzles through the LDS crossbar).
#include "itq3s_dev.h"
#include <atomic>

#include "itq3s_kernels.h"

namespace itq3s {

constexpr double kAblTStar = 0.7979;  // optimal ternary scale / sigma (Sec. 3.3, App. A)

template <int MASK>
__device__ __forceinline__ double abl_xor_f64(double v) {
    return row_xor_f64<MASK>(v);
}

// butterfly stage across lanes: the lower lane of a pair gets u + v, the upper one (-v) + u = u - v
// (one fused multiply-add with +-1: the product is exact)
template <int MASK>
__device__ __forceinline__ void abl_cross_stage(double (&a)[16], int lane) {
    const double sign = (lane & MASK) ? -1.0 : 1.0;
#pragma unroll
    for (int i = 0; i < 16; ++i) a[i] = __builtin_fma(a[i], sign, abl_xor_f64<MASK>(a[i]));  // (+-a) + p, one rounding
}

template <int L>  // lanes per block
__device__ __forceinline__ void abl_fwht(double (&a)[16], int lane) {
#pragma unroll
    for (int s = 1; s < 16; s <<= 1)
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if ((i & s) == 0) {
                const double u = a[i], v = a[i + s];
                a[i] = u + v;
                a[i + s] = u - v;
            }
    if constexpr (L > 1) abl_cross_stage<1>(a, lane);
    if constexpr (L > 2) abl_cross_stage<2>(a, lane);
    if constexpr (L > 4) abl_cross_stage<4>(a, lane);
    if constexpr (L > 8) abl_cross_stage<8>(a, lane);
    if constexpr (L > 16) abl_cross_stage<16>(a, lane);
}

// pairwise sum over the block: neighbours first, then distance 2, 4, ...; all lanes of the block agree
template <int L>
__device__ __forceinline__ double abl_block_sum(const double (&v)[16]) {
    double t[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) t[i] = v[2 * i] + v[2 * i + 1];
#pragma unroll
    for (int i = 0; i < 4; ++i) t[i] = t[2 * i] + t[2 * i + 1];
    t[0] = t[0] + t[1];
    t[1] = t[2] + t[3];
    double s = t[0] + t[1];
    if constexpr (L > 1) s = s + abl_xor_f64<1>(s);
    if constexpr (L > 2) s = s + abl_xor_f64<2>(s);
    if constexpr (L > 4) s = s + abl_xor_f64<4>(s);
    if constexpr (L > 8) s = s + abl_xor_f64<8>(s);
    if constexpr (L > 16) s = s + abl_xor_f64<16>(s);
    return s;
}

struct AblArgs {
    const float* W;
    uint8_t* codes;    // [N][K] or null
    uint32_t* scales;  // [N][K/n] or null
    float* What;       // [N][ldo] or null
    double* err;       // [2] or null: += sum (w_hat - w)^2, += sum w^2
    uint32_t* flags;
    int64_t N, K, ldw, ldo;
    int chunks;        // ceil(K / 1024)
    double cn;
};

template <int L>
__global__ __launch_bounds__(256) void roundtrip_kernel(const AblArgs a) {
    constexpr int n = 16 * L;
    __shared__ double red[2][4];
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int64_t total = a.N * a.chunks;  // (row, 1024-channel chunk) pairs, one per wavefront pass
    double se = 0.0, sw = 0.0;             // this lane's error sums over all its passes
    uint32_t my_flags = 0;
    for (int64_t id = (int64_t)blockIdx.x * 4 + wave; id < total; id += (int64_t)gridDim.x * 4) {
    const int64_t row = id / a.chunks;
    const int chunk = (int)(id - row * a.chunks);
    const int64_t k0 = (int64_t)chunk * 1024 + 16 * lane;
    const bool live = k0 < a.K;  // K is a multiple of n: a block is live or not as a whole
    const float4* src = reinterpret_cast<const float4*>(a.W + row * a.ldw + (live ? k0 : 0));
    const float4 w0 = src[0], w1 = src[1], w2 = src[2], w3 = src[3];
    const float wf[16] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w, w2.x, w2.y, w2.z, w2.w, w3.x, w3.y, w3.z, w3.w};
    double v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = (double)wf[i];
    abl_fwht<L>(v, lane);
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = v[i] * a.cn;
    const double mu = abl_block_sum<L>(v) / (double)n;
    double e2[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const double e = v[i] - mu;
        e2[i] = e * e;
    }
    const double sigma = sqrt(abl_block_sum<L>(e2) / (double)n);
    // a non-finite weight makes every transformed value of its block, hence the deviation, non-finite;
    // finite weights cannot (|w'| <= sqrt(n) * 3.4e38): one test per block instead of one per weight
    const bool block_bad = !(__builtin_fabs(sigma) <= 1.7976931348623157e308);
    double d64 = kAblTStar * sigma;
    bool sat = false, zclamp = false;
    if (d64 > 65504.0) { d64 = 65504.0; sat = true; }
    const _Float16 dh = (_Float16)(float)d64;
    const double d = (double)dh;
    const bool ok = !block_bad && d > 0.0;  // otherwise the block is stored as zeros
    const double rnd = floor(mu / (ok ? d : 1.0) + 0.5);
    double z = 0.0 - rnd;
    if (z > 2048.0) { z = 2048.0; zclamp = true; }
    if (z < -2048.0) { z = -2048.0; zclamp = true; }
    const double t_hi = (0.5 - z) * d, t_lo = (-0.5 - z) * d;
    uint32_t c[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) c[i] = ok ? (v[i] >= t_hi ? 2u : (v[i] < t_lo ? 0u : 1u)) : 1u;
    if (live) {
        if (block_bad) my_flags |= kFlagNonFinite;
        else if (sat) my_flags |= kFlagScaleSat;
        if (ok && zclamp) my_flags |= kFlagZClamp;
    }

    // ---- reconstruction: integer-valued butterflies (exact), one scaling
    double m[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) m[i] = ok ? ((double)((int)c[i] - 1) - z) : 0.0;
    abl_fwht<L>(m, lane);
    float wh[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const double r = (d * m[i]) * a.cn;
        wh[i] = (float)(ok ? r : 0.0);
        const double x = (double)wf[i], diff = (double)wh[i] - x;
        if (live && !block_bad) {
            se += diff * diff;
            sw += x * x;
        }
    }

    if (live) {
        if (a.codes != nullptr) {
            uint32_t pk[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) pk[q] = c[4 * q] | (c[4 * q + 1] << 8) | (c[4 * q + 2] << 16) | (c[4 * q + 3] << 24);
            *reinterpret_cast<uint4*>(a.codes + row * a.K + k0) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        }
        if (a.scales != nullptr && (lane & (L - 1)) == 0) {
            const _Float16 zh = (_Float16)(float)z;
            a.scales[row * (a.K / n) + k0 / n] =
                ok ? ((uint32_t)__builtin_bit_cast(uint16_t, dh) | ((uint32_t)__builtin_bit_cast(uint16_t, zh) << 16)) : 0u;
        }
        if (a.What != nullptr) {
            float4* dst = reinterpret_cast<float4*>(a.What + row * a.ldo + k0);
            dst[0] = make_float4(wh[0], wh[1], wh[2], wh[3]);
            dst[1] = make_float4(wh[4], wh[5], wh[6], wh[7]);
            dst[2] = make_float4(wh[8], wh[9], wh[10], wh[11]);
            dst[3] = make_float4(wh[12], wh[13], wh[14], wh[15]);
        }
    }
    }  // passes

    // one pair of additions per workgroup, one OR per wavefront
    if (a.err != nullptr) {
#pragma unroll
        for (int k = 1; k < 64; k <<= 1) {
            se += xor_lane_f64(se, k);
            sw += xor_lane_f64(sw, k);
        }
        if (lane == 0) {
            red[0][wave] = se;
            red[1][wave] = sw;
        }
        __syncthreads();
        if (threadIdx.x < 2) {
            const double t = (red[threadIdx.x][0] + red[threadIdx.x][1]) + (red[threadIdx.x][2] + red[threadIdx.x][3]);
            if ((int64_t)blockIdx.x * 4 < total) atomicAdd(a.err + threadIdx.x, t);
        }
    }
    if (a.flags != nullptr && __builtin_amdgcn_ballot_w64(my_flags != 0u) != 0ull) {
        uint32_t f = my_flags;
#pragma unroll
        for (int k = 1; k < 64; k <<= 1) f |= (uint32_t)__shfl_xor((int)f, k, 64);
        if (lane == 0) atomicOr(a.flags, f);
    }
}

static int compute_units() {
    static std::atomic<int> n_cached{0};
    int n = n_cached.load(std::memory_order_relaxed);
    if (n == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) n = v;
        else n = 256;
        n_cached.store(n, std::memory_order_relaxed);
    }
    return n;
}

// Grid: as many workgroups as the chip holds at once (what the register file allows per compute
// unit), each wavefront walking over its share of the (row, chunk) pairs.
template <int L>
static int launch_roundtrip_n(const AblArgs& a, hipStream_t stream) {
    static std::atomic<int> per_cu_cached{0};
    int per_cu = per_cu_cached.load(std::memory_order_relaxed);
    if (per_cu == 0) {
        int v = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&v, roundtrip_kernel<L>, 256, 0) != hipSuccess || v < 1) v = 2;
        per_cu = v;
        per_cu_cached.store(v, std::memory_order_relaxed);
    }
    const int64_t wgs = (a.N * a.chunks + 3) / 4, cap = (int64_t)per_cu * compute_units();
    hipLaunchKernelGGL(roundtrip_kernel<L>, dim3((unsigned)(wgs < cap ? wgs : cap)), dim3(256), 0, stream, a);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

int launch_roundtrip(const float* W, int64_t N, int64_t K, int64_t ldw, int n, uint8_t* codes, uint32_t* scales, float* What, int64_t ldo,
                     double* err, uint32_t* flags, hipStream_t stream) {
    AblArgs a;
    a.W = W; a.codes = codes; a.scales = scales; a.What = What; a.err = err; a.flags = flags;
    a.N = N; a.K = K; a.ldw = ldw; a.ldo = ldo; a.chunks = (int)((K + 1023) / 1024);
    switch (n) {  // c_n = 1/sqrt(n) to the nearest fp64
        case 32: a.cn = 0.17677669529663687; return launch_roundtrip_n<2>(a, stream);
        case 64: a.cn = 0.125; return launch_roundtrip_n<4>(a, stream);
        case 128: a.cn = 0.08838834764831843; return launch_roundtrip_n<8>(a, stream);
        case 256: a.cn = 0.0625; return launch_roundtrip_n<16>(a, stream);
        case 512: a.cn = 0.044194173824159216; return launch_roundtrip_n<32>(a, stream);
        default: return -2;
    }
}

}  // namespace itq3s
