// Activation-side rotation.  H is symmetric and its own inverse (Sec. 2.3), hence
//   <H v, x> = <v, H x>:
// instead of transforming every weight block, each 256-channel chunk of the activations is
// transformed once per call and the ternary digits are contracted with the rotated chunk.
//
// One wavefront per (row m, chunk b).  The 256-point transform runs on the matrix cores: with the
// chunk written as a 16 x 16 matrix X[a][b] = x[16a + b], the Sylvester construction gives
// H_256 = H_16 (x) H_16, i.e. (H x)[16a' + b'] = (H_16 X H_16)[a'][b'] / 16 (H_16 with entries +-1).
// T = X (H_16/4) is one 16x16x16 product (fp16 inputs, exact products, fp32 sums; the factor keeps
// |T| <= 4 max|x| inside the fp16 range); H_16 T follows with T split into two halves
// (T = T_hi + T_lo keeps 22 bits), then the remaining factor 1/4 and one rounding to fp16.  The
// accumulator layout of the first product is the B-operand layout of the second, so nothing moves
// between lanes.
#include "itq3s_dev.h"
#include "itq3s_kernels.h"

namespace itq3s {

// x~ = H x for one chunk.  Lane l reads x[16 (l%16) + 4 (l/16) + 0..3] and returns the rounded
// elements e = 64 (l/16) + 16 i + l%16, i = 0..3.
// Returns false if a rotated value (or the intermediate T, which then turns the result into NaN)
// leaves the fp16 range.
// `first` receives x[16 (l%16) + 4 (l/16)], the first of the lane's four inputs (lane 0: x[0]).
__device__ __forceinline__ bool rotate_chunk(const _Float16* __restrict__ src, int lane, _Float16 out[4], _Float16* first = nullptr) {
    const int r16 = lane & 15, g = lane >> 4;
    half4 h, q;  // H_16[4g + j][r16] and a quarter of it
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const bool neg = (__builtin_popcount((4 * g + j) & r16) & 1) != 0;
        h[j] = neg ? (_Float16)(-1.0f) : (_Float16)1.0f;
        q[j] = neg ? (_Float16)(-0.25f) : (_Float16)0.25f;
    }
    const half4 xa = *reinterpret_cast<const half4*>(src + 16 * r16 + 4 * g);
    if (first != nullptr) *first = xa[0];
    const floatx4 zero = {0.f, 0.f, 0.f, 0.f};
    const floatx4 T = __builtin_amdgcn_mfma_f32_16x16x16f16(xa, q, zero, 0, 0, 0);
    half4 th, tl;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        th[j] = (_Float16)T[j];
        tl[j] = (_Float16)(T[j] - (float)th[j]);
    }
    floatx4 U = __builtin_amdgcn_mfma_f32_16x16x16f16(h, th, zero, 0, 0, 0);
    U = __builtin_amdgcn_mfma_f32_16x16x16f16(h, tl, U, 0, 0, 0);
    bool ok = true;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        out[i] = (_Float16)(U[i] * 0.25f);
        ok = ok && __builtin_fabsf(U[i]) <= 4.0f * 65504.0f;  // (false for NaN as well)
    }
    return ok;
}

// Operand order of the streaming kernel.  The 16x16x32 MFMA of step t (0..7) takes from lane
// (column m, k-group g) eight halves; position i of those eight is element
//     e = 64 g + 16 (t>>1) + 4 (t&1) + (i>>1) + 8 (i&1)
// of the chunk, which is where the weight kernel's shift-and-mask unpack puts the code of the same
// element.  Xt index = (((b*8 + t)*4 + g)*MP + m)*8 + i.   S[b*MP + m] = sum_e x~_e (rounded values),
// S[KB*MP + b*MP + m] = 16 x_0 (the same sum before rounding, exact).
// (at least two wavefronts per SIMD: with a register budget of 256 the matrix instructions write ordinary
// vector registers; with the full 512 the compiler parks their results in accumulator registers and copies
// every one of them out)
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void rotate_frag_kernel(const _Float16* __restrict__ X, int64_t M, int64_t K, int64_t ldx, int MP,
                                                          _Float16* __restrict__ Xt, float* __restrict__ S, uint32_t* __restrict__ flags) {
    const int KB = (int)(K / kBlock);
    const int lane = lane_id();
    // (32-bit, wave-uniform index arithmetic: MP * KB chunks, far below 2^31)
    const int chunk = (int)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));  // m * KB + b over MP rows
    if (chunk >= MP * KB) return;
    const int m = chunk / KB, b = chunk - m * KB;
    _Float16 r[4] = {(_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f};
    _Float16 x0 = (_Float16)0.f;
    if (m < M && !rotate_chunk(X + (int64_t)m * ldx + (int64_t)b * kBlock, lane, r, &x0) && flags != nullptr) atomicOr(flags, kFlagActRange);
    // sum of the rounded chunk: inside a row of 16 lanes through the crossbar, the four rows through scalar registers
    float s = ((float)r[0] + (float)r[1]) + ((float)r[2] + (float)r[3]);
    s += __builtin_bit_cast(float, row_xor_i32<1>(__builtin_bit_cast(int, s)));
    s += __builtin_bit_cast(float, row_xor_i32<2>(__builtin_bit_cast(int, s)));
    s += __builtin_bit_cast(float, row_xor_i32<4>(__builtin_bit_cast(int, s)));
    s += __builtin_bit_cast(float, row_xor_i32<8>(__builtin_bit_cast(int, s)));
    const float total = (__builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, s), 0)) +
                         __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, s), 16))) +
                        (__builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, s), 32)) +
                         __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, s), 48)));
    if (lane == 0) {
        S[b * MP + m] = total;
        // exact sum of the unrounded chunk: H 1 = 16 e_0 (lane 0 holds x[0] from its operand load)
        S[KB * MP + b * MP + m] = 16.0f * (float)x0;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int e = 64 * (lane >> 4) + 16 * j + (lane & 15);
        const int g = e >> 6, w = (e >> 4) & 3, slot = e & 15;
        const int t = 2 * w + ((slot & 7) >> 2);
        const int i = 2 * (slot & 3) + (slot >> 3);
        Xt[(((((int64_t)b * 8 + t) * 4 + g) * MP + m) * 8) + i] = r[j];
    }
}

// Operand order of the tiled kernel: rows stay rows; inside every group of 16 channels, slot s moves
// to position 2 (s & 7) + (s >> 3), the order in which the tile loader's unpack emits the weights.
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void rotate_rowmajor_kernel(const _Float16* __restrict__ X, int64_t M, int64_t K, int64_t ldx,
                                                              _Float16* __restrict__ Xt, uint32_t* __restrict__ zero_words, int n_zero, uint32_t* __restrict__ flags) {
    const int64_t KB = K / kBlock;
    const int lane = lane_id();
    // the split-K flags of the contraction that follows start from zero
    if (blockIdx.x == 0)
        for (int i = threadIdx.x; i < n_zero; i += 256) zero_words[i] = 0u;
    const int64_t chunk = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (chunk >= M * KB) return;
    const int64_t m = chunk / KB, b = chunk - m * KB;
    _Float16 r[4];
    if (!rotate_chunk(X + m * ldx + b * kBlock, lane, r) && flags != nullptr) atomicOr(flags, kFlagActRange);
    _Float16* dst = Xt + m * K + b * kBlock;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int e = 64 * (lane >> 4) + 16 * j + (lane & 15), s = e & 15;
        dst[(e & ~15) | (2 * (s & 7) + (s >> 3))] = r[j];
    }
}

int launch_rotate_frag(const _Float16* X, int64_t M, int64_t K, int64_t ldx, int MP, _Float16* Xt, float* S, uint32_t* flags, hipStream_t stream) {
    const int64_t chunks = (int64_t)MP * (K / kBlock);
    hipLaunchKernelGGL(rotate_frag_kernel, dim3((unsigned)((chunks + 3) / 4)), dim3(256), 0, stream, X, M, K, ldx, MP, Xt, S, flags);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

int launch_rotate_rowmajor(const _Float16* X, int64_t M, int64_t K, int64_t ldx, _Float16* Xt, uint32_t* zero_words, int n_zero, uint32_t* flags,
                           hipStream_t stream) {
    const int64_t chunks = M * (K / kBlock);
    hipLaunchKernelGGL(rotate_rowmajor_kernel, dim3((unsigned)((chunks + 3) / 4)), dim3(256), 0, stream, X, M, K, ldx, Xt, zero_words, n_zero, flags);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

}  // namespace itq3s
