// Streaming matmul for M <= 16 activation rows (the decode path, Sec. 5.4).
//
//   Y[m][n] = sum_b d[n,b] * ( sum_j c[n,b,j] x~[m,b,j]  -  (1 + z[n,b]) * S[m,b] )
//
// with c = q+1 the stored code, x~ = H x the rotated activation chunk and S[m,b] = sum_j x~[m,b,j]
// (so that sum_j (c-1-z) x~ is formed without ever touching a signed digit).  The packed weights are
// read exactly once, with one 16-byte + one 8-byte + one 16-byte (scales) load per lane and tile;
// nothing dequantized is written anywhere.
//
// Contraction: v_mfma_f32_16x16x32_f16.  A operand = 16 weight rows of a tile, B operand = x~ for up
// to 16 activation rows.  A code c in {0,1,2} placed in bits 11:10 of a half is the number
// c * 2^-14 (bit pattern c<<10: exponent field 0, 1, 2, mantissa 0), so two codes that sit 16 bits
// apart in a low-plane word become a half2 with one shift and one mask; the factor 2^14 is applied
// to the block sum together with d.
//
// Work split: the grid is persistent, workgroup g owns a contiguous range of 16-row tiles and all of
// K; inside a workgroup, wavefront w takes blocks b = w, w+W, ... of a staged chunk of x~, keeps the
// B fragments of one block in registers and streams the (up to RT) row tiles of the current
// sub-group past them.  Loads for the next D steps are in flight while the current one is multiplied
// (ring of D+1 register buffers, main loop unrolled D+1 times so that every index is static).
#include "itq3s_dev.h"
#include "itq3s_kernels.h"

namespace itq3s {

constexpr int kGemvWaves = 8;                // wavefronts per workgroup
constexpr int kChunkBytesMax = 64 * 1024;    // x~ chunk staged in LDS

struct GemvArgs {
    const uint32_t* codes;
    const uint32_t* scales;
    const _Float16* Xt;  // rotated activations, operand order, MP columns
    const float* S;      // [KB][MP]
    void* Y;
    uint32_t* flags;
    int64_t N, ldy;
    int NT, KB, KC, M, y_f16;
};

struct TileRegs {
    u32x4 lo;
    u32x2 hi;
    u32x4 sc;
};

__device__ __forceinline__ void load_tile(TileRegs& r, const uint32_t* __restrict__ codes, const uint32_t* __restrict__ scales,
                                          int64_t tile, int lane) {
    const uint32_t* t = codes + tile * kTileWords;
    r.lo = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(t) + lane);
    r.hi = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(t + kTileLoWords) + lane);
    r.sc = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(scales + tile * kTileRows) + (lane >> 4));
}

__device__ __forceinline__ half8 as_half8(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
    u32x4 u = {a, b, c, d};
    return __builtin_bit_cast(half8, u);
}

// 64 codes of this lane (one tile row, one quarter of the block) times the matching x~ fragments.
__device__ __forceinline__ floatx4 tile_dot(const u32x4& lo, const half8 (&Bf)[8]) {
    constexpr uint32_t kMask = 0x0C000C00u;
    const uint32_t w[4] = {lo.x, lo.y, lo.z, lo.w};
    floatx4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t v = w[i];
        // slots j and j+8 of the word -> bits 11:10 and 27:26
        half8 a0 = as_half8((v << 10) & kMask, (v << 8) & kMask, (v << 6) & kMask, (v << 4) & kMask);
        half8 a1 = as_half8((v << 2) & kMask, v & kMask, (v >> 2) & kMask, (v >> 4) & kMask);
        c = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0, Bf[2 * i], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1, Bf[2 * i + 1], c, 0, 0, 0);
    }
    return c;
}

template <int MP, int RT, int D, int W>
__global__ __launch_bounds__(W * 64) void gemv_kernel(const GemvArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int KC = a.KC, KB = a.KB;
    _Float16* xs = reinterpret_cast<_Float16*>(smem);                                  // KC * MP * 256 halves
    float* ss = reinterpret_cast<float*>(smem + (size_t)KC * MP * 512);                // KC * MP floats
    float* red = reinterpret_cast<float*>(smem + (size_t)KC * MP * 512 + (((size_t)KC * MP * 4 + 15) & ~(size_t)15));  // W*256 floats

    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int g = lane >> 4, mcol = lane & 15, mm = mcol & (MP - 1);
    const int nt_begin = (int)(((int64_t)blockIdx.x * a.NT) / gridDim.x);
    const int nt_end = (int)(((int64_t)(blockIdx.x + 1) * a.NT) / gridDim.x);
    const int n_sg = (nt_end - nt_begin + RT - 1) / RT;
    const int n_chunks = (KB + KC - 1) / KC;
    if (n_sg == 0) return;

    // Step = (sub-group sg, chunk c, j): this wavefront's block b = c*KC + j*W + wave (if inside the
    // chunk) against row tiles nt_begin + sg*RT + [0, RT).  Every wavefront runs the same number of
    // steps so that the barriers below line up.
    struct Step {
        int sg, c, j;
    };
    auto steps_in_chunk = [&](int c) { return (min(KC, KB - c * KC) + W - 1) / W; };
    auto advance = [&](Step& s) {
        if (++s.j == steps_in_chunk(s.c)) {
            s.j = 0;
            if (++s.c == n_chunks) { s.c = 0; ++s.sg; }
        }
    };
    auto issue = [&](const Step& s, TileRegs (&buf)[RT]) {
        if (s.sg >= n_sg) return;
        const int b = s.c * KC + s.j * W + wave;
        if (b >= min((s.c + 1) * KC, KB)) return;
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            const int nt = nt_begin + s.sg * RT + rt;
            if (nt < nt_end) load_tile(buf[rt], a.codes, a.scales, (int64_t)nt * KB + b, lane);
        }
    };

    floatx4 acc[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) acc[rt] = floatx4{0.f, 0.f, 0.f, 0.f};
    uint32_t bad = 0;

    // x~ chunk c (and its S values): global -> registers, then registers -> LDS between two barriers.
    constexpr int kStageMax = kChunkBytesMax / (W * 64 * 16);
    u32x4 stage[kStageMax];
#pragma unroll
    for (int i = 0; i < kStageMax; ++i) stage[i] = u32x4{0u, 0u, 0u, 0u};
    float stage_s = 0.f;
    auto stage_load = [&](int c) {
        const int c_len = min(KC, KB - c * KC);
        const u32x4* src = reinterpret_cast<const u32x4*>(a.Xt + (size_t)c * KC * MP * 256);
        const int n16 = c_len * MP * 32;  // 16-byte units
#pragma unroll
        for (int i = 0; i < kStageMax; ++i) {
            const int idx = i * (W * 64) + threadIdx.x;
            if (idx < n16) stage[i] = src[idx];
        }
        if ((int)threadIdx.x < c_len * MP) stage_s = a.S[(size_t)c * KC * MP + threadIdx.x];
    };
    auto stage_publish = [&](int c) {
        const int c_len = min(KC, KB - c * KC);
        const int n16 = c_len * MP * 32;
        __syncthreads();  // everyone is done with the previous chunk
#pragma unroll
        for (int i = 0; i < kStageMax; ++i) {
            const int idx = i * (W * 64) + threadIdx.x;
            if (idx < n16) reinterpret_cast<u32x4*>(xs)[idx] = stage[i];
        }
        if ((int)threadIdx.x < c_len * MP) ss[threadIdx.x] = stage_s;
        __syncthreads();
    };

    auto run_step = [&](const Step& s, const Step& ahead, const TileRegs (&cur)[RT], TileRegs (&nxt)[RT], bool first) {
        // the very first chunk is staged before the loop; later chunks (only when x~ does not fit
        // in one chunk) are staged here, loads issued ahead of the prefetch
        const bool new_chunk = s.j == 0 && n_chunks > 1 && !first;
        const int c_len = min(KC, KB - s.c * KC);
        if (new_chunk) stage_load(s.c);
        issue(ahead, nxt);  // prefetch the step D ahead into the buffer that was consumed last
        if (new_chunk) stage_publish(s.c);
        // (d) multiply
        const int bl = s.j * W + wave;
        if (bl < c_len) {
            half8 Bf[8];
#pragma unroll
            for (int t = 0; t < 8; ++t)
                Bf[t] = *reinterpret_cast<const half8*>(xs + ((size_t)((bl * 8 + t) * 4 + g) * MP + mm) * 8);
            const float sv = ss[bl * MP + mm];
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                const int nt = nt_begin + s.sg * RT + rt;
                if (nt < nt_end) {
                    const TileRegs& tr = cur[rt];
                    const floatx4 c = tile_dot(tr.lo, Bf);
                    bad |= tr.hi.x | tr.hi.y;
                    const uint32_t sw[4] = {tr.sc.x, tr.sc.y, tr.sc.z, tr.sc.w};
                    const uint32_t zbits = (sw[0] | sw[1] | sw[2] | sw[3]) >> 16;
                    if (__builtin_amdgcn_ballot_w64(zbits != 0u) == 0ull) {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            acc[rt][i] = __builtin_fmaf(f16_bits_to_f32(sw[i] & 0xffffu), __builtin_fmaf(c[i], 16384.0f, -sv), acc[rt][i]);
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float zf = 1.0f + f16_bits_to_f32(sw[i] >> 16);
                            acc[rt][i] = __builtin_fmaf(f16_bits_to_f32(sw[i] & 0xffffu), __builtin_fmaf(c[i], 16384.0f, -(zf * sv)), acc[rt][i]);
                        }
                    }
                }
            }
        }
        // (e) end of a sub-group: add the W partial sums, store Y
        if (s.c == n_chunks - 1 && s.j == steps_in_chunk(s.c) - 1) {
            constexpr int kPerRound = 16 / MP;  // row tiles per round through the 16 KB reduction buffer
#pragma unroll
            for (int r0 = 0; r0 < RT; r0 += kPerRound) {
                __syncthreads();
#pragma unroll
                for (int rr = 0; rr < kPerRound; ++rr) {
                    const int rt = r0 + rr;
                    if (rt < RT && mcol < MP) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) red[((wave * kPerRound + rr) * 16 + 4 * g + i) * MP + mcol] = acc[rt][i];
                    }
                }
                __syncthreads();
                // outputs of this round: kPerRound tiles x 16 rows x MP columns; thread -> (m, rr, row)
                for (int o = threadIdx.x; o < kPerRound * 16 * MP; o += W * 64) {
                    const int row = o & 15, rr = (o >> 4) % kPerRound, m = o / (16 * kPerRound);
                    const int rt = r0 + rr;
                    const int nt = nt_begin + s.sg * RT + rt;
                    const int64_t n = (int64_t)nt * 16 + row;
                    if (rt < RT && nt < nt_end && n < a.N && m < a.M) {
                        float sum = 0.f;
#pragma unroll
                        for (int wv = 0; wv < W; ++wv) sum += red[((wv * kPerRound + rr) * 16 + row) * MP + m];
                        if (a.y_f16) reinterpret_cast<_Float16*>(a.Y)[m * a.ldy + n] = (_Float16)sum;
                        else reinterpret_cast<float*>(a.Y)[m * a.ldy + n] = sum;
                    }
                }
            }
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) acc[rt] = floatx4{0.f, 0.f, 0.f, 0.f};
        }
    };

    constexpr int NB = D + 1;
    TileRegs ring[NB][RT];
    Step s{0, 0, 0}, ahead{0, 0, 0};
    stage_load(0);
#pragma unroll
    for (int k = 0; k < D; ++k) {
        issue(ahead, ring[k]);
        advance(ahead);
    }
    stage_publish(0);
    bool done = false, first = true;
    while (!done) {
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            if (!done) {
                run_step(s, ahead, ring[k], ring[(k + D) % NB], first);
                first = false;
                advance(s);
                advance(ahead);
                done = s.sg >= n_sg;
            }
        }
    }
    if (a.flags != nullptr && bad != 0u) atomicOr(a.flags, kFlagBadCode);
}

template <int MP, int RT, int D, int W>
static int launch_one(const GemvArgs& a, int grid, size_t lds, hipStream_t stream) {
    auto kern = gemv_kernel<MP, RT, D, W>;
    static bool lds_limit_raised = false;  // once per instantiation: allow up to the 160 KB of a CU
    if (!lds_limit_raised) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) return -6;
        lds_limit_raised = true;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(W * 64), lds, stream, a);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

static int cu_count() {
    static int n = 0;
    if (n == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) n = v;
        else n = 256;
    }
    return n;
}

template <int MP>
static int launch_mp(GemvArgs a, hipStream_t stream) {
    constexpr int W = kGemvWaves;
    // chunk of x~ kept in LDS
    const int kc_cap = kChunkBytesMax / (MP * 512);
    a.KC = a.KB < kc_cap ? a.KB : kc_cap;
    const size_t lds = (size_t)a.KC * MP * 512 + (((size_t)a.KC * MP * 4 + 15) & ~(size_t)15) + (size_t)W * 256 * 4;
    const int grid = a.NT < cu_count() ? a.NT : cu_count();
    // row tiles per workgroup decide how many tiles one step covers; keep about 8 tiles in flight
    const int per_wg = (a.NT + grid - 1) / grid;
    if (per_wg <= 1) return launch_one<MP, 1, 8, W>(a, grid, lds, stream);
    if (per_wg == 2) return launch_one<MP, 2, 4, W>(a, grid, lds, stream);
    if (per_wg == 3) return launch_one<MP, 3, 3, W>(a, grid, lds, stream);
    return launch_one<MP, 4, 2, W>(a, grid, lds, stream);
}

int launch_gemv(const uint32_t* codes, const uint32_t* scales, int64_t N, int64_t K, const _Float16* Xt, const float* S, int64_t M,
                int MP, void* Y, int y_f16, int64_t ldy, uint32_t* flags, hipStream_t stream) {
    GemvArgs a;
    a.codes = codes; a.scales = scales; a.Xt = Xt; a.S = S; a.Y = Y; a.flags = flags;
    a.N = N; a.ldy = ldy; a.NT = (int)((N + 15) / 16); a.KB = (int)(K / kBlock); a.KC = 0; a.M = (int)M; a.y_f16 = y_f16;
    switch (MP) {
        case 1: return launch_mp<1>(a, stream);
        case 2: return launch_mp<2>(a, stream);
        case 4: return launch_mp<4>(a, stream);
        case 8: return launch_mp<8>(a, stream);
        case 16: return launch_mp<16>(a, stream);
    }
    return -2;
}

}  // namespace itq3s
