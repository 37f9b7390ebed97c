// Activation-side rotation.  H is symmetric and its own inverse (Sec. 2.3), hence
//   <H v, x> = <v, H x>:
// instead of transforming every weight block, each 256-channel chunk of the activations is
// transformed once per call and the ternary digits are contracted with the rotated chunk.
//
// One wavefront per (row m, chunk b); lane l holds elements 4l..4l+3 in fp32, butterflies as in the
// weight-side kernels, one rounding to fp16 at the end.
#include "itq3s_dev.h"
#include "itq3s_kernels.h"

namespace itq3s {

// x~ = H x for one chunk; returns the four rounded values of this lane.
__device__ __forceinline__ void rotate_chunk(const _Float16* __restrict__ src, int lane, _Float16 out[4]) {
    const half4 h = *reinterpret_cast<const half4*>(src + 4 * lane);
    float v0 = (float)h[0], v1 = (float)h[1], v2 = (float)h[2], v3 = (float)h[3];
    float t0 = v0 + v1, t1 = v0 - v1, t2 = v2 + v3, t3 = v2 - v3;
    v0 = t0 + t2; v2 = t0 - t2; v1 = t1 + t3; v3 = t1 - t3;
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) {
        const bool upper = (lane & m) != 0;
        const float p0 = xor_lane_f32(v0, m), p1 = xor_lane_f32(v1, m), p2 = xor_lane_f32(v2, m), p3 = xor_lane_f32(v3, m);
        v0 = upper ? (p0 - v0) : (v0 + p0);
        v1 = upper ? (p1 - v1) : (v1 + p1);
        v2 = upper ? (p2 - v2) : (v2 + p2);
        v3 = upper ? (p3 - v3) : (v3 + p3);
    }
    out[0] = (_Float16)(v0 * 0.0625f);
    out[1] = (_Float16)(v1 * 0.0625f);
    out[2] = (_Float16)(v2 * 0.0625f);
    out[3] = (_Float16)(v3 * 0.0625f);
}

// Operand order of the streaming kernel.  The 16x16x32 MFMA of step t (0..7) takes from lane
// (column m, k-group g) eight halves; position i of those eight is element
//     e = 64 g + 16 (t>>1) + 4 (t&1) + (i>>1) + 8 (i&1)
// of the chunk, which is where the weight kernel's shift-and-mask unpack puts the code of the same
// element.  Xt index = (((b*8 + t)*4 + g)*MP + m)*8 + i.   S[b*MP + m] = sum_e x~_e (rounded values).
__global__ __launch_bounds__(256) void rotate_frag_kernel(const _Float16* __restrict__ X, int64_t M, int64_t K, int64_t ldx, int MP,
                                                          _Float16* __restrict__ Xt, float* __restrict__ S) {
    const int64_t KB = K / kBlock;
    const int lane = lane_id();
    const int64_t chunk = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // m * KB + b over MP rows
    if (chunk >= (int64_t)MP * KB) return;
    const int64_t m = chunk / KB, b = chunk - m * KB;
    _Float16 r[4] = {(_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f};
    if (m < M) rotate_chunk(X + m * ldx + b * kBlock, lane, r);
    float s = ((float)r[0] + (float)r[1]) + ((float)r[2] + (float)r[3]);
#pragma unroll
    for (int k = 1; k < 64; k <<= 1) s += xor_lane_f32(s, k);
    if (lane == 0) S[b * MP + m] = s;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int e = 4 * lane + j;
        const int g = e >> 6, w = (e >> 4) & 3, slot = e & 15;
        const int t = 2 * w + ((slot & 7) >> 2);
        const int i = 2 * (slot & 3) + (slot >> 3);
        Xt[((((b * 8 + t) * 4 + g) * MP + m) * 8) + i] = r[j];
    }
}

// Operand order of the tiled kernel: rows stay rows; inside every group of 16 channels, slot s moves
// to position 2 (s & 7) + (s >> 3), the order in which the tile loader's unpack emits the weights.
__global__ __launch_bounds__(256) void rotate_rowmajor_kernel(const _Float16* __restrict__ X, int64_t M, int64_t K, int64_t ldx,
                                                              _Float16* __restrict__ Xt) {
    const int64_t KB = K / kBlock;
    const int lane = lane_id();
    const int64_t chunk = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (chunk >= M * KB) return;
    const int64_t m = chunk / KB, b = chunk - m * KB;
    _Float16 r[4];
    rotate_chunk(X + m * ldx + b * kBlock, lane, r);
    _Float16* dst = Xt + m * K + b * kBlock;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int e = 4 * lane + j, s = e & 15;
        dst[(e & ~15) | (2 * (s & 7) + (s >> 3))] = r[j];
    }
}

int launch_rotate_frag(const _Float16* X, int64_t M, int64_t K, int64_t ldx, int MP, _Float16* Xt, float* S, hipStream_t stream) {
    const int64_t chunks = (int64_t)MP * (K / kBlock);
    hipLaunchKernelGGL(rotate_frag_kernel, dim3((unsigned)((chunks + 3) / 4)), dim3(256), 0, stream, X, M, K, ldx, MP, Xt, S);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

int launch_rotate_rowmajor(const _Float16* X, int64_t M, int64_t K, int64_t ldx, _Float16* Xt, hipStream_t stream) {
    const int64_t chunks = M * (K / kBlock);
    hipLaunchKernelGGL(rotate_rowmajor_kernel, dim3((unsigned)((chunks + 3) / 4)), dim3(256), 0, stream, X, M, K, ldx, Xt);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

}  // namespace itq3s
