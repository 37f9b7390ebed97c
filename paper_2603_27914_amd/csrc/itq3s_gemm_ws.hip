// Tiled matmul with the rotation on the WEIGHT side, as the paper's kernel does it (Alg. 2): every
// 256-channel block of a weight tile is unpacked, scaled and passed through the inverse transform on
// its way into on-chip memory, and the matrix cores multiply the un-rotated activations with the
// reconstructed fp16 weights.  No dequantized weight reaches HBM.
//
//   Y[m][n] = sum_k x[m][k] * w_hat[n][k],   w_hat = H( d (q - z) )   rounded once to fp16
//
// The library's default path rotates the activations instead (itq3s_gemm.hip); this kernel exists to
// measure what the weight-side placement costs on this machine: the transform work is repeated for
// every 128-row slab of activations that meets the weight tile.
//
// Workgroup: 256 threads = 2 x 2 wavefronts, tile 128 (m) x 128 (n) x 256 (k = one block), wavefront
// tile 64 x 64 as 2 x 2 v_mfma_f32_32x32x16_f16.  Per block step the workgroup copies a 128 x 256
// slab of X into LDS and reconstructs 128 weight rows: a wavefront takes one row at a time, each lane
// extracts its four codes, and two 16x16x16 products give the transposed 256-point transform
// (H_256 = H_16 (x) H_16, all integers exact), leaving every lane with four consecutive channels;
// the zero-point reaches only channel 0 (H 1 = 16 e_0), in fp32 before the rounding.
#include <hip/hip_ext.h>

#include "itq3s_dev.h"
#include <atomic>

#include "itq3s_kernels.h"

namespace itq3s {

constexpr int WM = 128, WN = 128, WK = 256;
constexpr int WLD = WK + 8;                     // LDS row stride in halves (528 bytes: 16-byte reads conflict-free)
constexpr int kGemmWsLds = 2 * WM * WLD * 2;    // bytes: X slab + weight slab

struct GemmWsArgs {
    const uint32_t* codes;
    const uint32_t* scales;
    const _Float16* X;  // [M][ldx], not rotated
    void* Y;
    uint32_t* flags;
    int64_t N, M, ldx, ldy;
    int NT, KB, y_f16;
};

// (at least two wavefronts per SIMD: with a register budget of 256 the matrix instructions write ordinary
// vector registers; with the full 512 the compiler parks their results in accumulator registers and copies
// every one of them out)
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void gemm_ws_kernel(const GemmWsArgs a) {
    extern __shared__ __align__(16) _Float16 lds[];
    _Float16* const As = lds;             // [WM][WLD] activations
    _Float16* const Bs = lds + WM * WLD;  // [WN][WLD] reconstructed weights

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, kg = lane >> 5;
    const int r16 = lane & 15, g = lane >> 4;
    const int64_t m0 = (int64_t)blockIdx.y * WM;
    const int64_t n0 = (int64_t)blockIdx.x * WN;

    half4 h;  // H_16[4g + j][r16]: B operand of the first product, A operand of the second
#pragma unroll
    for (int j = 0; j < 4; ++j) h[j] = (__builtin_popcount((4 * g + j) & r16) & 1) ? (_Float16)(-1.0f) : (_Float16)1.0f;

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    bool bad = false;

    for (int b = 0; b < a.KB; ++b) {
        __syncthreads();  // the previous step's fragments have been read
        // ---- activations: 128 rows x 256 channels, 16-byte pieces (row = idx/32, piece = idx%32)
#pragma unroll 4
        for (int i = 0; i < 16; ++i) {
            const int idx = tid + 256 * i, row = idx >> 5, c = idx & 31;
            const int64_t m = m0 + row;
            const uint4 v = m < a.M ? *reinterpret_cast<const uint4*>(a.X + m * a.ldx + (int64_t)b * kBlock + c * 8) : make_uint4(0, 0, 0, 0);
            *reinterpret_cast<uint4*>(&As[row * WLD + c * 8]) = v;
        }
        // ---- weights: wavefront w reconstructs rows 32w .. 32w+31 of the tile, one row per pass
#pragma unroll 4
        for (int rr = 0; rr < 32; ++rr) {
            const int row = wave * 32 + rr;
            const int64_t n = n0 + row;
            half4 o = {(_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f};
            if (n < a.N) {  // wavefront-uniform
                const int64_t tile = (n >> 4) * a.KB + b;
                const int r = (int)(n & 15);
                const uint32_t* t = a.codes + tile * kTileWords;
                // channels e = 64 g + 16 j + r16 (j = 0..3) sit in slot r16 of low-plane word j of storage
                // lane 16 g + r; their high bits in bit 16 (j & 1) + r16 of high-plane word j >> 1
                const u32x4 lo = *reinterpret_cast<const u32x4*>(t + 4 * (16 * g + r));
                const u32x2 hi = *reinterpret_cast<const u32x2*>(t + kTileLoWords + 2 * (16 * g + r));
                const uint32_t sw = a.scales[tile * kTileRows + r];
                const uint32_t lw[4] = {lo.x, lo.y, lo.z, lo.w};
                const uint32_t hw[2] = {hi.x, hi.y};
                half4 v;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t c = (lw[j] >> (2 * r16)) & 3u;
                    bad |= ((hw[j >> 1] >> (16 * (j & 1) + r16)) & 1u) != 0u;
                    v[j] = (_Float16)(float)((int)c - 1);
                }
                const floatx4 zero = {0.f, 0.f, 0.f, 0.f};
                const floatx4 T = __builtin_amdgcn_mfma_f32_16x16x16f16(v, h, zero, 0, 0, 0);  // V^T H_16
                const half4 th = {(_Float16)T[0], (_Float16)T[1], (_Float16)T[2], (_Float16)T[3]};
                const floatx4 U = __builtin_amdgcn_mfma_f32_16x16x16f16(h, th, zero, 0, 0, 0);  // channels 16 r16 + 4 g + 0..3
                const float d = f16_bits_to_f32(sw & 0xffffu);
                const float z = f16_bits_to_f32(sw >> 16);
                float f[4] = {U[0], U[1], U[2], U[3]};
                if (lane == 0) f[0] = f[0] - 256.0f * z;  // H_u applied to the constant -z
#pragma unroll
                for (int i = 0; i < 4; ++i) o[i] = (_Float16)((d * f[i]) * 0.0625f);
            }
            *reinterpret_cast<half4*>(&Bs[row * WLD + 16 * r16 + 4 * g]) = o;
        }
        __syncthreads();
        // ---- 16 MFMA steps over the block
#pragma unroll 4
        for (int ks = 0; ks < WK / 16; ++ks) {
            half8 af[2], bf[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) af[i] = *reinterpret_cast<const half8*>(&As[(wm * 64 + i * 32 + l32) * WLD + ks * 16 + kg * 8]);
#pragma unroll
            for (int j = 0; j < 2; ++j) bf[j] = *reinterpret_cast<const half8*>(&Bs[(wn * 64 + j * 32 + l32) * WLD + ks * 16 + kg * 8]);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
    }

    // accumulator register v of a 32x32 block: row = 8*(v/4) + 4*(lane/32) + v%4, column = lane%32
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int64_t n = n0 + wn * 64 + j * 32 + l32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t m = m0 + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
                if (m < a.M && n < a.N) {
                    if (a.y_f16) reinterpret_cast<_Float16*>(a.Y)[m * a.ldy + n] = (_Float16)acc[i][j][v];
                    else reinterpret_cast<float*>(a.Y)[m * a.ldy + n] = acc[i][j][v];
                }
            }
        }
    if (a.flags != nullptr && __builtin_amdgcn_ballot_w64(bad) != 0ull && lane == 0) atomicOr(a.flags, kFlagBadCode);
}

int launch_gemm_weight_side(const uint32_t* codes, const uint32_t* scales, int64_t N, int64_t K, const _Float16* X, int64_t ldx, int64_t M,
                            void* Y, int y_f16, int64_t ldy, uint32_t* flags, hipStream_t stream) {
    GemmWsArgs a;
    a.codes = codes; a.scales = scales; a.X = X; a.Y = Y; a.flags = flags;
    a.N = N; a.M = M; a.ldx = ldx; a.ldy = ldy; a.NT = (int)((N + 15) / 16); a.KB = (int)(K / kBlock); a.y_f16 = y_f16;
    static std::atomic<bool> lds_limit_raised{false};
    if (!lds_limit_raised) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_ws_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kGemmWsLds) != hipSuccess) return -6;
        lds_limit_raised = true;
    }
    const dim3 grid((unsigned)((N + WN - 1) / WN), (unsigned)((M + WM - 1) / WM));
    const LaunchTiming tm = take_launch_timing();
    if (tm.start != nullptr) hipExtLaunchKernelGGL(gemm_ws_kernel, grid, dim3(256), kGemmWsLds, stream, tm.start, tm.stop, 0, a);
    else hipLaunchKernelGGL(gemm_ws_kernel, grid, dim3(256), kGemmWsLds, stream, a);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

}  // namespace itq3s
