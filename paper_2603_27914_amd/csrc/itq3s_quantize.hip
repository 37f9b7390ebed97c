// Offline quantizer (Alg. 1, Def. 1) in fp64, every operation in a fixed order so that the packed
// output is bit-identical on any IEEE-754 machine.
//
// A block (256 consecutive channels of one row) is held by eight lanes, 32 consecutive elements
// each; a wavefront = one workgroup covers eight rows of a 16-row storage tile.  Butterfly stages
// with distance 1 .. 16 stay inside the lane; distances 32, 64 and 128 exchange with lanes l^1, l^2,
// l^4 through the LDS crossbar (swizzles: no memory access).  What every lane of a block computes
// redundantly (the tails of two pairwise sums, a square root, a division, the scale and zero-point)
// is spread over 32 elements.  The 32 codes of a lane are two low-plane words of one storage lane:
// one 8-byte store from registers.  Each lane reads its 128 contiguous bytes (one cache line) with
// eight 16-byte loads issued back to back.  This file must be compiled with floating point
// contraction off: every add, subtract and multiply below rounds on its own.
#include "itq3s_dev.h"
#include "itq3s_kernels.h"

namespace itq3s {

constexpr double kTStar = 0.7979;  // optimal ternary scale / sigma (Sec. 3.3, App. A)

// Pairwise sums in the oracle's order: neighbours first, then distance 2, 4, ... inside the lane
// (written as a tree so that no array of squares is ever held), then the remaining distances across
// the lanes of the block.  Addition is commutative bit for bit, so every lane ends with the same value.
template <int E, int LO, int HI>
__device__ __forceinline__ double lane_tree_sum(const double (&v)[E]) {
    if constexpr (HI - LO == 1) return v[LO];
    else return lane_tree_sum<E, LO, (LO + HI) / 2>(v) + lane_tree_sum<E, (LO + HI) / 2, HI>(v);
}
template <int E, int LO, int HI>
__device__ __forceinline__ double lane_tree_sq(const double (&v)[E], double mu) {
    if constexpr (HI - LO == 1) {
        const double e = v[LO] - mu;
        return e * e;
    } else return lane_tree_sq<E, LO, (LO + HI) / 2>(v, mu) + lane_tree_sq<E, (LO + HI) / 2, HI>(v, mu);
}
template <int LB>
__device__ __forceinline__ double block_lanes_sum(double s) {  // over the LB lanes of a block
    s = s + row_xor_f64<1>(s);
    s = s + row_xor_f64<2>(s);
    if constexpr (LB > 4) s = s + row_xor_f64<4>(s);
    return s;
}
// One cross-lane butterfly stage: the lower lane of a pair gets u + v, the upper one u - v (u the
// lower lane's value).  Both are one fused multiply-add (+-1) * own + other: the product is exact,
// so the upper lane's (-v) + u is u - v bit for bit.
template <int E, int MASK>
__device__ __forceinline__ void cross_stage(double (&a)[E], int h) {
    const double sign = (h & MASK) ? -1.0 : 1.0;
#pragma unroll
    for (int i = 0; i < E; ++i) a[i] = __builtin_fma(a[i], sign, row_xor_f64<MASK>(a[i]));
}

// E = elements per lane (32 or 64), LB = 256 / E lanes per block, 64 / LB rows per wavefront: half a
// tile (E = 32, grid = 2 tiles) or a whole one (E = 64, grid = tiles).  Measured on 4096x4096 /
// 11008x4096 / 28672x8192: 3.8 / 4.7 / 5.0 TB/s with 32 (110 registers, four wavefronts per SIMD),
// 3.2 / 3.8 / 4.7 with 64 (168 registers, three per SIMD, and wavefronts so long that a tensor fills
// the chip only a few times over); 16 elements per lane, the first version, ran at 3.3 / 3.6 / 4.3.
// kSub: the sub-block-scale variant of the format (Sec. 4.1: 8 fp16 sub-scales per block, 116 bytes).
// A lane of the E = 32 arrangement holds exactly one sub-block (32 consecutive rotated coefficients), so
// its deviation about the block mean is the lane's own partial of the pairwise sum; the sub-scale is
// s_j = T* sigma_j / d (rounded to fp16 through fp32 like d), the digit thresholds become
// (+-0.5 s_j - z) d, and d, z are those of the base format.  Lanes 2g, 2g+1 of a block share one
// storage word: subscales[tile*64 + 16 g + r] = s_2g | s_(2g+1) << 16.
template <int E, bool kSub>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(E == 64 ? 3 : 4))) void quantize_kernel(
    const float* __restrict__ W, int64_t N, int64_t K, int64_t ldw, uint32_t* __restrict__ codes, uint32_t* __restrict__ scales,
    uint32_t* __restrict__ subscales, uint32_t* __restrict__ flags, int KB) {
    static_assert(E == 32 || E == 64, "elements per lane");
    static_assert(!kSub || E == 32, "a lane must hold one sub-block");
    constexpr int LB = kBlock / E, RW = 64 / LB, PARTS = kTileRows / RW, WPL = E / 16;  // WPL low-plane words per lane
    const int tile = (int)(blockIdx.x / PARTS), part = (int)(blockIdx.x % PARTS);  // tile = nt * KB + b
    const int nt = tile / KB, b = tile - nt * KB;
    const int lane = lane_id();
    const int r = part * RW + lane / LB, h = lane % LB;  // row of the tile; elements E h .. E h + E - 1 of its block
    const int64_t n = (int64_t)nt * kTileRows + r;
    uint32_t* const out = codes + (int64_t)tile * kTileWords;

    // high plane: always 0 on encode (128 words per tile, shared out over its wavefronts)
    if constexpr (PARTS == 1) *reinterpret_cast<u32x2*>(out + kTileLoWords + 2 * lane) = u32x2{0u, 0u};
    else out[kTileLoWords + 64 * part + lane] = 0u;

    uint32_t my_flags = 0;
    uint32_t word[WPL];
#pragma unroll
    for (int i = 0; i < WPL; ++i) word[i] = 0x55555555u;  // codes "1" = digit 0
    uint32_t scale_word = 0u;
    uint32_t sub_bits = 0u;
    if (n < N) {  // (uniform over the lanes of a block; the moves below never leave them)
        double a[E];
        const float4* src = reinterpret_cast<const float4*>(W + n * ldw + (int64_t)b * kBlock + E * h);
        float4 in[E / 4];
#pragma unroll
        for (int k = 0; k < E / 4; ++k) in[k] = src[k];
#pragma unroll
        for (int k = 0; k < E / 4; ++k) {
            const float4 f = in[k];
            const float wf[4] = {f.x, f.y, f.z, f.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) a[4 * k + j] = (double)wf[j];
        }

        // w' = H w: stages below E in registers (the lower index gets u+v, the higher one u-v) ...
#pragma unroll
        for (int s = 1; s < E; s <<= 1)
#pragma unroll
            for (int i = 0; i < E; ++i)
                if ((i & s) == 0) {
                    const double u = a[i], v = a[i + s];
                    a[i] = u + v;
                    a[i + s] = u - v;
                }
        // ... stages E .. 128 across the lanes of the block
        cross_stage<E, 1>(a, h);
        cross_stage<E, 2>(a, h);
        if constexpr (LB > 4) cross_stage<E, 4>(a, h);
        // a = 16 w' from here on.  The factor 1/16 of the normalised transform is a power of two: it
        // commutes with every rounding below (nothing comes near the ends of the fp64 range: |a| < 2^136
        // and squares of fp32-derived values stay above 2^-300), so it is applied to the few block
        // scalars instead of the elements, with bit-identical results.
        const double sum16 = block_lanes_sum<LB>(lane_tree_sum<E, 0, E>(a));
        const double mu = sum16 / 4096.0;                                                                     // mean of w'
        const double lane_sq = lane_tree_sq<E, 0, E>(a, sum16 / 256.0);  // 256 x the squared deviations of the lane's coefficients
        const double sigma = sqrt(block_lanes_sum<LB>(lane_sq) / 65536.0);  // deviation of w'
        // a non-finite weight makes every transformed value, hence the deviation, non-finite; finite
        // weights cannot (|w'| <= 16 * 3.4e38)
        const bool row_bad = !(__builtin_fabs(sigma) <= 1.7976931348623157e308);
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
        double step = 1.0;  // digit step in units of d
        if constexpr (kSub) {
            double s64 = kTStar * sqrt(lane_sq / 8192.0) / (live ? d : 1.0);  // T* sigma_j / d, sigma_j over the lane's 32 coefficients
            if (s64 > 65504.0) { s64 = 65504.0; sat = true; }
            const _Float16 sh = (_Float16)(float)s64;
            step = (double)sh;
            if (live) sub_bits = (uint32_t)__builtin_bit_cast(uint16_t, sh);
        }
        const double t_hi = (0.5 * step - z) * d * 16.0, t_lo = (-0.5 * step - z) * d * 16.0;  // exact products; against a = 16 w'
        if (live && !(step > 0.0)) {
            // (sub-block variant only) a sub-scale of zero: digit 0 everywhere in the sub-block
            const _Float16 zh = (_Float16)(float)z;
            scale_word = (uint32_t)__builtin_bit_cast(uint16_t, dh) | ((uint32_t)__builtin_bit_cast(uint16_t, zh) << 16);
            if (zclamp) my_flags |= kFlagZClamp;
        } else if (live) {
#pragma unroll
            for (int i = 0; i < WPL; ++i) word[i] = 0u;
#pragma unroll
            for (int i = 0; i < E; ++i) {
                const uint32_t c = a[i] >= t_hi ? 2u : (a[i] < t_lo ? 0u : 1u);
                word[i >> 4] |= c << (2 * (i & 15));
            }
            const _Float16 zh = (_Float16)(float)z;
            scale_word = (uint32_t)__builtin_bit_cast(uint16_t, dh) | ((uint32_t)__builtin_bit_cast(uint16_t, zh) << 16);
            if (zclamp) my_flags |= kFlagZClamp;
        }
        if (row_bad) my_flags |= kFlagNonFinite;
        else if (sat) my_flags |= kFlagScaleSat;
    }
    // elements E h .. E h + E - 1 of row r: low-plane words (E h / 16) % 4 .. of storage lane 16 (E h / 64) + r
    uint32_t* const dst = out + 4 * (16 * (E * h / 64) + r) + (E * h / 16) % 4;
    if constexpr (WPL == 4) *reinterpret_cast<u32x4*>(dst) = u32x4{word[0], word[1], word[2], word[3]};
    else *reinterpret_cast<u32x2*>(dst) = u32x2{word[0], word[1]};
    if (h == 0) scales[(int64_t)tile * kTileRows + r] = scale_word;
    if constexpr (kSub) {
        const uint32_t other = (uint32_t)row_xor_i32<1>((int)sub_bits);  // the neighbouring sub-block's scale
        if ((h & 1) == 0) subscales[(int64_t)tile * 64 + 16 * (h >> 1) + r] = sub_bits | (other << 16);
    }
    if (flags != nullptr && __builtin_amdgcn_ballot_w64(my_flags != 0u) != 0ull) {
        // one atomic per wavefront: OR of the flags of its lanes
        uint32_t f = my_flags;
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) f |= (uint32_t)__shfl_xor((int)f, m, 64);
        if (lane == 0) atomicOr(flags, f);
    }
}

int launch_quantize(const float* W, int64_t N, int64_t K, int64_t ldw, uint32_t* codes, uint32_t* scales, uint32_t* subscales, uint32_t* flags,
                    hipStream_t stream) {
    const int64_t tiles = ((N + 15) / 16) * (K / kBlock);
    if (tiles > 0x3fffffff) return -2;
    if (subscales != nullptr)
        hipLaunchKernelGGL((quantize_kernel<32, true>), dim3((unsigned)(2 * tiles)), dim3(64), 0, stream, W, N, K, ldw, codes, scales, subscales, flags, (int)(K / kBlock));
    else
        hipLaunchKernelGGL((quantize_kernel<32, false>), dim3((unsigned)(2 * tiles)), dim3(64), 0, stream, W, N, K, ldw, codes, scales, subscales, flags, (int)(K / kBlock));
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

}  // namespace itq3s
