// Tiled matmul with the rotation on the WEIGHT side, as the paper's kernel does it (Alg. 2): every
// 256-channel block of a weight tile is unpacked, scaled and passed through the inverse transform on
// its way into on-chip memory, and the matrix cores multiply the un-rotated activations with the
// reconstructed fp16 weights.  No dequantized weight reaches HBM.
//
//   Y[m][n] = sum_k x[m][k] * w_hat[n][k],   w_hat = H( d (q - z) )   rounded once to fp16
//
// The library's default path rotates the activations instead (itq3s_gemm.hip); this kernel exists to
// measure what the weight-side placement costs on this machine when it is done as well as the
// placement allows: a reconstructed weight tile stays in LDS and is multiplied with as many
// activation rows as one workgroup's accumulators can hold.
//
// Workgroup: 512 threads = 4 (m) x 2 (n) wavefronts, tile 512 (m) x 128 (n), K in blocks of 256;
// wavefront tile 128 x 64 = 4 x 2 v_mfma_f32_32x32x16_f16 (128 accumulator registers).  The
// transform of a 128 x 256 weight tile is thus shared by 512 activation rows (it is repeated
// ceil(M / 512) times in all; for M <= 512 exactly once).
//
// Per block:  (1) every wavefront reconstructs one 16-row storage tile into the LDS weight tile.  Its
// packed words -- loaded one block ahead, 28 bytes per lane -- go through a wavefront-private LDS
// stage, from which the 16 lanes of a group read row r's words by broadcast; per row, every lane
// extracts its four codes and two 16x16x16 products give the transposed 256-point transform
// (H_256 = H_16 (x) H_16, all integers exact), leaving every lane with four consecutive channels; the
// zero-point reaches only channel 0 (H 1 = 16 e_0), in fp32 before the one rounding to fp16.  Four
// rows run as independent chains.  (2) eight steps of 32 channels: the activations of a step
// (512 x 32) are loaded two steps ahead into registers and parked in one of two LDS buffers, one
// barrier per step.  The reconstruction is not overlapped with the products of another block: what
// it costs is what the placement costs.
#include <hip/hip_ext.h>

#include "itq3s_dev.h"
#include <atomic>

#include "itq3s_kernels.h"

namespace itq3s {

constexpr int WM = 512, WN = 128, WK = 256, WSTEP = 32;
constexpr int WLD = WK + 8;                   // weight tile row stride in halves (528 bytes: 16-byte reads conflict-free)
constexpr int XLD = WSTEP + 8;                // activation buffer row stride in halves (80 bytes)
constexpr int kWsStageWords = 352;            // per wavefront: 256 low-plane words, 16 x (d / 16, 256 z) as floats, 64 sub-scale words
constexpr int kWsBsBytes = WN * WLD * 2;      // 67584
constexpr int kWsAsBytes = WM * XLD * 2;      // 40960 per buffer
constexpr int kGemmWsLds = kWsBsBytes + 2 * kWsAsBytes + 8 * kWsStageWords * 4;  // 160768 of 163840

struct GemmWsArgs {
    const uint32_t* codes;
    const uint32_t* scales;
    const uint32_t* subscales;  // the 116-byte variant's sub-scale array (kSub)
    const _Float16* X;  // [M][ldx], not rotated
    void* Y;
    uint32_t* flags;
    int64_t N, M, ldx, ldy;
    int NT, KB, y_f16;
};

// kSub: the sub-block-scale variant (Sec. 4.1): the digit of channel j of the rotated block is multiplied by
// the fp16 scale of its sub-block (j / 32) before the transform; the products are exact halves, their
// 16-term sums T are not, so T goes into the second product as two halves (22 bits) and that product
// takes two matrix instructions instead of one.
template <bool kSub>
__global__ __launch_bounds__(512) void gemm_ws_kernel(const GemmWsArgs a) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    _Float16* const Bs = reinterpret_cast<_Float16*>(lds_raw);                       // [WN][WLD] reconstructed weights of the block
    _Float16* const As = reinterpret_cast<_Float16*>(lds_raw + kWsBsBytes);          // [2][WM][XLD] activations of a step
    uint32_t* const stage_all = reinterpret_cast<uint32_t*>(lds_raw + kWsBsBytes + 2 * kWsAsBytes);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, kg = lane >> 5;
    const int r16 = lane & 15, g = lane >> 4;
    const int64_t m0 = (int64_t)blockIdx.y * WM;
    const int64_t n0 = (int64_t)blockIdx.x * WN;
    uint32_t* const stage = stage_all + wave * kWsStageWords;

    half4 h;  // H_16[4g + j][r16]: B operand of the first product, A operand of the second
#pragma unroll
    for (int j = 0; j < 4; ++j) h[j] = (__builtin_popcount((4 * g + j) & r16) & 1) ? (_Float16)(-1.0f) : (_Float16)1.0f;

    // the wavefront's storage tile: rows n0 + 16 wave ..; a tile beyond the tensor is read from the last
    // valid one and scaled by zero
    const int my_tile = (int)(n0 >> 4) + wave;
    const bool tile_ok = my_tile < a.NT;
    const int64_t tile_base = (int64_t)(tile_ok ? my_tile : a.NT - 1) * a.KB;

    // activations: thread t carries pieces t, t + 512, t + 1024, t + 1536 of a step (piece = 16 bytes; four per row)
    const _Float16* xp[4];
    bool xok[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int idx = tid + 512 * i, row = idx >> 2, c = idx & 3;
        const int64_t m = m0 + row;
        xok[i] = m < a.M;
        xp[i] = a.X + (xok[i] ? m : 0) * a.ldx + c * 8;
    }
    const int total_steps = a.KB * (WK / WSTEP);
    auto load_x = [&](int s, uint4 (&xr)[4]) {
        const int64_t koff = (int64_t)(s < total_steps ? s : total_steps - 1) * WSTEP;
#pragma unroll
        for (int i = 0; i < 4; ++i) xr[i] = xok[i] ? *reinterpret_cast<const uint4*>(xp[i] + koff) : make_uint4(0, 0, 0, 0);
    };
    auto park_x = [&](int s, const uint4 (&xr)[4]) {
        _Float16* const dst = As + (s & 1) * (WM * XLD);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = tid + 512 * i, row = idx >> 2, c = idx & 3;
            *reinterpret_cast<uint4*>(&dst[row * XLD + c * 8]) = xr[i];
        }
    };
    u32x4 t_lo;
    u32x2 t_hi;
    uint32_t t_sc, t_ss = 0u;
    auto load_tile = [&](int b) {
        const int64_t tile = tile_base + (b < a.KB ? b : a.KB - 1);
        const uint32_t* t = a.codes + tile * kTileWords;
        t_lo = *reinterpret_cast<const u32x4*>(t + 4 * lane);
        t_hi = *reinterpret_cast<const u32x2*>(t + kTileLoWords + 2 * lane);
        t_sc = tile_ok ? a.scales[tile * kTileRows + r16] : 0u;
        if constexpr (kSub) t_ss = a.subscales[tile * 64 + lane];
    };

    floatx16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    bool bad = false;

    uint4 xr[2][4];  // activations of the next two steps on their way to LDS
    load_tile(0);
    load_x(0, xr[1]);
    park_x(0, xr[1]);
    load_x(1, xr[1]);

    for (int b = 0; b < a.KB; ++b) {
        // ---- (1) reconstruct the wavefront's 16 rows of block b (everybody has left the previous block's products:
        //          the barrier behind its last step)
        *reinterpret_cast<u32x4*>(stage + 4 * lane) = t_lo;
        if (lane < 16) {  // row r16's factors, once per tile: d / 16 (a power of two: commutes with every rounding) and 256 z
            const float d16 = f16_bits_to_f32(t_sc & 0xffffu) * 0.0625f;
            *reinterpret_cast<float2*>(stage + 256 + 2 * lane) = make_float2(d16, 256.0f * f16_bits_to_f32(t_sc >> 16));
        }
        if constexpr (kSub) stage[288 + lane] = t_ss;
        bad |= tile_ok && (t_hi.x | t_hi.y) != 0u;
        load_tile(b + 1);
#pragma unroll 4
        for (int rr = 0; rr < 16; ++rr) {
            // channels e = 64 g + 16 j + r16 (j = 0..3) sit in slot r16 of low-plane word j of storage lane 16 g + rr
            const u32x4 lo = *reinterpret_cast<const u32x4*>(stage + 4 * (16 * g + rr));
            const float2 dz = *reinterpret_cast<const float2*>(stage + 256 + 2 * rr);
            // two codes OR-ed into the mantissas of a pair of halves 1024.0, minus 1025: the digits c - 1, exact
            const uint32_t p0 = ((lo.x >> (2 * r16)) & 3u) | (((lo.y >> (2 * r16)) & 3u) << 16) | 0x64006400u;
            const uint32_t p1 = ((lo.z >> (2 * r16)) & 3u) | (((lo.w >> (2 * r16)) & 3u) << 16) | 0x64006400u;
            const half2v bias = {(_Float16)(-1025.0f), (_Float16)(-1025.0f)};
            const half2v v01 = __builtin_bit_cast(half2v, p0) + bias, v23 = __builtin_bit_cast(half2v, p1) + bias;
            half4 v = {v01[0], v01[1], v23[0], v23[1]};
            if constexpr (kSub) {  // channels 64 g + 16 j + r16: sub-block 2 g for j = 0, 1 and 2 g + 1 for j = 2, 3 (the two halves of the lane's word)
                const half2v s2 = __builtin_bit_cast(half2v, stage[288 + 16 * g + rr]);
                v = half4{v[0] * s2[0], v[1] * s2[0], v[2] * s2[1], v[3] * s2[1]};
            }
            const floatx4 zero = {0.f, 0.f, 0.f, 0.f};
            const floatx4 T = __builtin_amdgcn_mfma_f32_16x16x16f16(v, h, zero, 0, 0, 0);  // V^T H_16
            const half4 th = {(_Float16)T[0], (_Float16)T[1], (_Float16)T[2], (_Float16)T[3]};
            floatx4 U = __builtin_amdgcn_mfma_f32_16x16x16f16(h, th, zero, 0, 0, 0);  // channels 16 r16 + 4 g + 0..3
            if constexpr (kSub) {
                const half4 tl = {(_Float16)(T[0] - (float)th[0]), (_Float16)(T[1] - (float)th[1]), (_Float16)(T[2] - (float)th[2]), (_Float16)(T[3] - (float)th[3])};
                U = __builtin_amdgcn_mfma_f32_16x16x16f16(h, tl, U, 0, 0, 0);
            }
            const float f0 = lane == 0 ? U[0] - dz.y : U[0];  // H_u applied to the constant -z
            const half4 o = {(_Float16)(dz.x * f0), (_Float16)(dz.x * U[1]), (_Float16)(dz.x * U[2]), (_Float16)(dz.x * U[3])};
            *reinterpret_cast<half4*>(&Bs[(wave * 16 + rr) * WLD + 16 * r16 + 4 * g]) = o;
        }
        __syncthreads();  // the weight tile and the first step's activations are in place
        // ---- (2) eight steps of 32 channels
#pragma unroll 2
        for (int e = 0; e < WK / WSTEP; ++e) {
            const int s = b * (WK / WSTEP) + e;
            load_x(s + 2, xr[e & 1]);  // two steps ahead: a step's products are shorter than a load's way from memory
            const _Float16* const Ab = As + (s & 1) * (WM * XLD);
#pragma unroll
            for (int ks = 0; ks < WSTEP / 16; ++ks) {
                half8 af[4], bf[2];
#pragma unroll
                for (int i = 0; i < 4; ++i) af[i] = *reinterpret_cast<const half8*>(&Ab[(wm * 128 + i * 32 + l32) * XLD + ks * 16 + kg * 8]);
#pragma unroll
                for (int j = 0; j < 2; ++j) bf[j] = *reinterpret_cast<const half8*>(&Bs[(wn * 64 + j * 32 + l32) * WLD + e * WSTEP + ks * 16 + kg * 8]);
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
            }
            park_x(s + 1, xr[(e + 1) & 1]);  // the other buffer: its readers passed the barrier behind the previous step
            __syncthreads();
        }
    }

    // accumulator register v of a 32x32 block: row = 8*(v/4) + 4*(lane/32) + v%4, column = lane%32
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int64_t n = n0 + wn * 64 + j * 32 + l32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t m = m0 + wm * 128 + i * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
                if (m < a.M && n < a.N) {
                    if (a.y_f16) reinterpret_cast<_Float16*>(a.Y)[m * a.ldy + n] = (_Float16)acc[i][j][v];
                    else reinterpret_cast<float*>(a.Y)[m * a.ldy + n] = acc[i][j][v];
                }
            }
        }
    if (a.flags != nullptr && __builtin_amdgcn_ballot_w64(bad) != 0ull && lane == 0) atomicOr(a.flags, kFlagBadCode);
}

template <bool kSub>
static int launch_ws(const GemmWsArgs& a, dim3 grid, hipStream_t stream) {
    static std::atomic<bool> lds_limit_raised{false};
    if (!lds_limit_raised) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_ws_kernel<kSub>), hipFuncAttributeMaxDynamicSharedMemorySize, kGemmWsLds) != hipSuccess) return -6;
        lds_limit_raised = true;
    }
    const LaunchTiming tm = take_launch_timing();
    if (tm.start != nullptr) hipExtLaunchKernelGGL(gemm_ws_kernel<kSub>, grid, dim3(512), kGemmWsLds, stream, tm.start, tm.stop, 0, a);
    else hipLaunchKernelGGL(gemm_ws_kernel<kSub>, grid, dim3(512), kGemmWsLds, stream, a);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

int launch_gemm_weight_side(const uint32_t* codes, const uint32_t* scales, const uint32_t* subscales, int64_t N, int64_t K, const _Float16* X,
                            int64_t ldx, int64_t M, void* Y, int y_f16, int64_t ldy, uint32_t* flags, hipStream_t stream) {
    GemmWsArgs a;
    a.codes = codes; a.scales = scales; a.subscales = subscales; a.X = X; a.Y = Y; a.flags = flags;
    a.N = N; a.M = M; a.ldx = ldx; a.ldy = ldy; a.NT = (int)((N + 15) / 16); a.KB = (int)(K / kBlock); a.y_f16 = y_f16;
    const dim3 grid((unsigned)((N + WN - 1) / WN), (unsigned)((M + WM - 1) / WM));
    return subscales != nullptr ? launch_ws<true>(a, grid, stream) : launch_ws<false>(a, grid, stream);
}

}  // namespace itq3s
