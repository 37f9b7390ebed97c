// Streaming matmul for 5 <= M <= 16 activation rows: a rotation launch (itq3s_rotate.hip) writes
// x~ = H x in operand order to the workspace, and this kernel streams the packed weights against
// those fragments.  Same sum, same contraction on v_mfma_f32_16x16x32_f16 and same storage walk as
// the kernel for M <= 4 (itq3s_gemv.hip), which rotates inside the kernel instead; see there for the
// formula.  Work split: workgroup g owns at most RT 16-row tiles and all of K; wavefront w takes
// blocks w, w+8, ...; tile loads and activation fragments run D blocks ahead through a ring of D+1
// register buffers; every pipelined load is issued unconditionally (steps past the end of a
// wavefront's list re-read tile 0) so that the load counter alone orders loads and use.
#include <hip/hip_ext.h>

#include "itq3s_dev.h"
#include <atomic>
#include <type_traits>

#include "itq3s_kernels.h"

namespace itq3s {
namespace rows {

constexpr int kGemvWaves = 8;        // wavefronts per workgroup
constexpr int kGemvMaxRT = 7;        // row tiles per workgroup, at most
// fused rotation: blocks per wavefront times MP, at most (bounds the registers and the LDS the rotated
// activations take, and the time every workgroup spends rotating the same activations)
// (32 for 8 and 16 rows was measured: slower than the separate rotation launch; for 2 to 4 rows it
// wins on long K: 4096x11008 at M = 4 12.0 -> 10.5 us, 8192x28672 at M = 2 28.2 -> 24.4 us)
constexpr int fused_max_blocks(int mp) { return mp <= 4 ? 32 : 16; }

// One launch serves up to kGemvMaxGroup weight tensors that share K and the activations (the
// projections of one layer that read the same input).  Their 16-row tiles are numbered as one list,
// tensor after tensor, and split evenly over the workgroups; a workgroup's tiles may belong to two
// tensors.
struct GemvTensor {
    const uint32_t* codes;
    const uint32_t* scales;
    void* Y;
    int64_t N, ldy;
    int v_begin;  // position of this tensor's first row tile in the list (0x7fffffff for unused entries)
    int pad_;
};

struct GemvArgs {
    GemvTensor t[kGemvMaxGroup];
    const _Float16* X;  // kFused: activations [M][ldx]; direct: rotated, operand order, MP columns
    const float* S;     // direct only: [KB][MP]
    uint32_t* flags;
    int64_t ldx;
    int KB, M, y_f16;
    int nt_q, nt_r;  // row tiles per workgroup: the first nt_r workgroups own nt_q + 1, the others nt_q
};

struct TileRegs {
    u32x4 lo;
    u32x2 hi;
    uint32_t sc;
};

__device__ __forceinline__ void load_tile(TileRegs& r, const uint32_t* __restrict__ codes, const uint32_t* __restrict__ scales,
                                          int64_t tile, int lane) {
    const uint32_t* t = codes + tile * kTileWords;
    r.lo = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(t) + lane);
    r.hi = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(t + kTileLoWords) + lane);
    r.sc = __builtin_nontemporal_load(scales + tile * kTileRows + (lane & 15));
}

__device__ __forceinline__ half8 as_half8(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
    u32x4 u = {a, b, c, d};
    return __builtin_bit_cast(half8, u);
}

// 64 codes of this lane (one tile row, one quarter of the block) against the matching x~ fragments:
// returns sum_j c_j 2^-14 x~[m][j] for m = 4*(lane/16) + 0..3 and the lane's weight row; the MFMA
// adds the four quarters of the block.
__device__ __forceinline__ floatx4 tile_dot(const u32x4& lo, const half8 (&Xf)[8]) {
    constexpr uint32_t kMask = 0x0C000C00u;
    const uint32_t w[4] = {lo.x, lo.y, lo.z, lo.w};
    floatx4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t v = w[i];
        // slots j and j+8 of the word -> bits 11:10 and 27:26
        half8 a0 = as_half8((v << 10) & kMask, (v << 8) & kMask, (v << 6) & kMask, (v << 4) & kMask);
        half8 a1 = as_half8((v << 2) & kMask, v & kMask, (v >> 2) & kMask, (v >> 4) & kMask);
        c = __builtin_amdgcn_mfma_f32_16x16x32_f16(Xf[2 * i], a0, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x32_f16(Xf[2 * i + 1], a1, c, 0, 0, 0);
    }
    return c;
}

// value of lane (l ^ MASK): data-parallel-primitive moves inside a row of 16 lanes, LDS crossbar
// (no memory access) across rows
template <int MASK>
__device__ __forceinline__ float lane_xor(float v) {
    int x = __builtin_bit_cast(int, v);
    if constexpr (MASK == 1) x = __builtin_amdgcn_update_dpp(x, x, 0xB1, 0xf, 0xf, false);       // quad_perm [1,0,3,2]
    else if constexpr (MASK == 2) x = __builtin_amdgcn_update_dpp(x, x, 0x4E, 0xf, 0xf, false);  // quad_perm [2,3,0,1]
    else if constexpr (MASK == 4) {  // l^7 (mirror in 8) then l^3 (reverse in 4)
        x = __builtin_amdgcn_update_dpp(x, x, 0x141, 0xf, 0xf, false);
        x = __builtin_amdgcn_update_dpp(x, x, 0x1B, 0xf, 0xf, false);
    } else if constexpr (MASK == 8) {  // l^15 (mirror in 16) then l^7
        x = __builtin_amdgcn_update_dpp(x, x, 0x140, 0xf, 0xf, false);
        x = __builtin_amdgcn_update_dpp(x, x, 0x141, 0xf, 0xf, false);
    } else x = __shfl_xor(x, MASK, 64);
    return __builtin_bit_cast(float, x);
}

// The 256-point transform on the matrix cores.  With the chunk written as a 16 x 16 matrix
// X[a][b] = x[16a + b], the Sylvester construction gives H_256 = H_16 (x) H_16, i.e.
//     (H x)[16a' + b'] = (H_16 X H_16)[a'][b'] / 16        (H_16 with entries +-1).
// Two 16x16x16 products do it: T = X (H_16/4) (fp16 inputs, exact products, fp32 sums; the factor
// keeps |T| <= 4 max|x| inside the fp16 range), then H_16 T with T split into two halves
// (T = T_hi + T_lo keeps 22 bits), then the remaining factor 1/4.  The accumulator layout of the
// first product (lane = column b', four rows a per lane) is exactly the B-operand layout of the
// second, so nothing moves between lanes.  A lane holds x[16 (l%16) + 4 (l/16) + 0..3] on entry and
// element e = 64 (l/16) + 16 r + l%16, r = 0..3, of the result.
struct HadamardOperand {
    half4 h, q;  // H_16[4g + j][r16] and a quarter of it, j = 0..3: B operand of the first product, A operand of the second
    __device__ __forceinline__ void init(int lane) {
        const int r16 = lane & 15, g = lane >> 4;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool neg = (__builtin_popcount((4 * g + j) & r16) & 1) != 0;
            h[j] = neg ? (_Float16)(-1.0f) : (_Float16)1.0f;
            q[j] = neg ? (_Float16)(-0.25f) : (_Float16)0.25f;
        }
    }
};

// x~ = H x for one 256-chunk, rounded to fp16, scattered into operand order at `dst` (256*MP halves:
// index ((t*4 + g)*MP + m)*8 + i); kSum: returns the sum of the rounded values in every lane.
template <int MP, bool kSum>
__device__ __forceinline__ float rotate_to_lds(u32x2 raw, const HadamardOperand& H, int lane, int m, _Float16* dst) {
    const half4 xa = __builtin_bit_cast(half4, raw);
    const floatx4 zero = {0.f, 0.f, 0.f, 0.f};
    const floatx4 T = __builtin_amdgcn_mfma_f32_16x16x16f16(xa, H.q, zero, 0, 0, 0);
    half4 th, tl;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        th[j] = (_Float16)T[j];
        tl[j] = (_Float16)(T[j] - (float)th[j]);
    }
    floatx4 U = __builtin_amdgcn_mfma_f32_16x16x16f16(H.h, th, zero, 0, 0, 0);
    U = __builtin_amdgcn_mfma_f32_16x16x16f16(H.h, tl, U, 0, 0, 0);
    _Float16 r[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = (_Float16)(U[i] * 0.25f);
    float s = 0.f;
    if constexpr (kSum) {
        s = ((float)r[0] + (float)r[1]) + ((float)r[2] + (float)r[3]);
        s += lane_xor<1>(s); s += lane_xor<2>(s); s += lane_xor<4>(s); s += lane_xor<8>(s); s += lane_xor<16>(s); s += lane_xor<32>(s);
    }
    // element e = 64g + 16w + slot (w = r, slot = l%16): quarter g, low-plane word w, code slot `slot`;
    // MFMA step t = 2w + ((slot&7)>>2), position i = 2(slot&3) + (slot>>3)
    const int g = lane >> 4, slot = lane & 15;
    const int tb = (slot & 7) >> 2, i0 = 2 * (slot & 3) + (slot >> 3);
#pragma unroll
    for (int w = 0; w < 4; ++w) dst[(((2 * w + tb) * 4 + g) * MP + m) * 8 + i0] = r[w];
    return s;
}

// NBX = 0: direct; NBX > 0: fused, with room for NBX blocks per wavefront (NBX * MP <= fused_max_blocks(MP)).
// kGrouped: the launch serves several tensors (a single-tensor launch skips the lookup and the
// fetch of the unused descriptors, which are on the way to the first load).
template <int MP, int RT, int D, int NBX, bool kGrouped>
__global__ __launch_bounds__(kGemvWaves * 64) void gemv_kernel(const GemvArgs a) {
    constexpr bool kFused = NBX > 0;
    // Several activation rows: the block sums S come from the matrix cores (the same fragments against an
    // operand of all ones, eight instructions per block on an otherwise idle pipe) instead of one
    // cross-lane sum per rotated chunk, and the rotations of a slot are straight-line code whose
    // dependent chains overlap.  One row: the cross-lane sum is cheaper (measured).
    constexpr bool kMfmaSum = MP >= 2;
    constexpr int W = kGemvWaves;
    constexpr int NB = D + 1;
    extern __shared__ __align__(16) unsigned char smem[];
    const int KB = a.KB;

    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));  // wave-uniform, in an SGPR
    const int g = lane >> 4, r16 = lane & 15, mm = r16 & (MP - 1);
    // 1..RT row tiles of the list (the host picks the grid that way); no division and no dependent
    // fetch on the way to the first load.  Per slot: the tile row's first tile in codes / scales; a
    // missing slot reads the first tile of the launch (never used).
    const int wg = (int)blockIdx.x;
    const int nt_begin = wg * a.nt_q + (wg < a.nt_r ? wg : a.nt_r);
    const int cnt = a.nt_q + (wg < a.nt_r ? 1 : 0);
    struct SlotOut {   // where the 16 outputs of a slot go (table in LDS, read back in the epilogue)
        void* Y;
        int64_t ldy;
        int64_t n0;    // first row of the tile inside its tensor
        int64_t rows;  // rows of that tensor from n0 on that exist (<= 0: slot unused)
    };
    SlotOut* const slot_out = reinterpret_cast<SlotOut*>(smem + (size_t)W * NBX * MP * (512 + 8) + (size_t)W * RT * MP * 16 * 4);
    const uint32_t* slot_codes[RT];
    const uint32_t* slot_scales[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        // tensor that owns list position nt_begin + rt (scalar selects; all descriptors come with the
        // first argument fetch)
        const uint32_t* t_codes = a.t[0].codes;
        const uint32_t* t_scales = a.t[0].scales;
        void* t_y = a.t[0].Y;
        int64_t t_n = a.t[0].N, t_ldy = a.t[0].ldy;
        int t_begin = 0;
        if constexpr (kGrouped) {
#pragma unroll
            for (int i = 1; i < kGemvMaxGroup; ++i) {
                const bool ge = nt_begin + rt >= a.t[i].v_begin;
                t_codes = ge ? a.t[i].codes : t_codes;
                t_scales = ge ? a.t[i].scales : t_scales;
                t_y = ge ? a.t[i].Y : t_y;
                t_n = ge ? a.t[i].N : t_n;
                t_ldy = ge ? a.t[i].ldy : t_ldy;
                t_begin = ge ? a.t[i].v_begin : t_begin;
            }
        }
        const int64_t local = nt_begin + rt - t_begin;
        const int64_t first = rt < cnt ? local * KB : 0;
        slot_codes[rt] = (rt < cnt ? t_codes : a.t[0].codes) + first * kTileWords;
        slot_scales[rt] = (rt < cnt ? t_scales : a.t[0].scales) + first * kTileRows;
        if (threadIdx.x == 0) slot_out[rt] = SlotOut{t_y, t_ldy, local * 16, rt < cnt ? t_n - local * 16 : 0};
    }
    const int nb = KB > wave ? (KB - wave + W - 1) / W : 0;  // blocks of this wavefront: b = wave + j*W

    // LDS: kFused: per wavefront NBX*MP*256 halves of x~, then per wavefront NBX*MP sums S and NBX*MP
    // sums E; then the reduction buffer
    _Float16* xs = reinterpret_cast<_Float16*>(smem) + (size_t)wave * NBX * MP * 256;
    float* ss = reinterpret_cast<float*>(smem + (size_t)W * NBX * MP * 512) + wave * NBX * MP * 2;
    float* se = ss + NBX * MP;
    float* red = reinterpret_cast<float*>(smem + (size_t)W * NBX * MP * (512 + 8));  // W*RT*MP*16 floats
    float* spare = reinterpret_cast<float*>(smem + (size_t)W * NBX * MP * (512 + 8) + (size_t)W * RT * MP * 16 * 4 + (size_t)RT * 32) + wave * 64;

    floatx4 acc[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) acc[rt] = floatx4{0.f, 0.f, 0.f, 0.f};
    uint32_t bad = 0;

    struct Slot {
        TileRegs t[RT];
        half8 xf[kFused ? 1 : 8];
        floatx4 sv, ev;
    };
    Slot ring[NB];

    // loads of step j (block wave + j*W against all row tiles of the workgroup); past the end of
    // the list, and for missing row tiles, tile 0 / block 0 stand in (never used)
    // Tiles [R0, R1) of step j.  The activations of the step (direct path) travel with the first part.
    auto issue_part = [&](Slot& s, int j, auto r0c, auto r1c) {
        constexpr int R0 = decltype(r0c)::value, R1 = decltype(r1c)::value;
        const bool live = j < nb;
        const int b = wave + j * W;
#pragma unroll
        for (int rt = R0; rt < R1; ++rt) load_tile(s.t[rt], slot_codes[rt], slot_scales[rt], live ? b : 0, lane);
        if constexpr (!kFused && R0 == 0) {
            const int bb = live ? b : 0;
#pragma unroll
            for (int t = 0; t < 8; ++t) s.xf[t] = *reinterpret_cast<const half8*>(a.X + ((size_t)((bb * 8 + t) * 4 + g) * MP + mm) * 8);
            const float* E = a.S + (size_t)KB * MP;
            if constexpr (MP >= 4) {
                s.sv = *reinterpret_cast<const floatx4*>(a.S + (size_t)bb * MP + ((4 * g) & (MP - 1)));
                s.ev = *reinterpret_cast<const floatx4*>(E + (size_t)bb * MP + ((4 * g) & (MP - 1)));
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    s.sv[i] = a.S[(size_t)bb * MP + ((4 * g + i) & (MP - 1))];
                    s.ev[i] = E[(size_t)bb * MP + ((4 * g + i) & (MP - 1))];
                }
            }
        }
    };
    auto issue = [&](Slot& s, int j) { issue_part(s, j, std::integral_constant<int, 0>{}, std::integral_constant<int, RT>{}); };

    struct StepOperands {
        half8 Xf[8];
        floatx4 sv, ev;
    };
    auto prepare = [&](StepOperands& o, const Slot& s, int j) {
        if constexpr (kFused) {
            const _Float16* xb = xs + (size_t)j * MP * 256;
#pragma unroll
            for (int t = 0; t < 8; ++t) o.Xf[t] = *reinterpret_cast<const half8*>(xb + ((t * 4 + g) * MP + mm) * 8);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if constexpr (!kMfmaSum) o.sv[i] = ss[j * MP + ((4 * g + i) & (MP - 1))];
                o.ev[i] = se[j * MP + ((4 * g + i) & (MP - 1))];
            }
        } else {
#pragma unroll
            for (int t = 0; t < 8; ++t) o.Xf[t] = s.xf[t];
            o.sv = s.sv;
            o.ev = s.ev;
        }
        if constexpr (kFused && kMfmaSum) {
            floatx4 sacc = {0.f, 0.f, 0.f, 0.f};
            const half8 ones = as_half8(0x04000400u, 0x04000400u, 0x04000400u, 0x04000400u);  // 2^-14 each
#pragma unroll
            for (int t = 0; t < 8; ++t) sacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(o.Xf[t], ones, sacc, 0, 0, 0);
#pragma unroll
            for (int i = 0; i < 4; ++i) o.sv[i] = sacc[i] * 16384.0f;
        }
    };
    auto compute_part = [&](const StepOperands& o, const Slot& s, auto r0c, auto r1c) {
        constexpr int R0 = decltype(r0c)::value, R1 = decltype(r1c)::value;
#pragma unroll
        for (int rt = R0; rt < R1; ++rt) {
            if (rt < cnt) {
                const TileRegs& tr = s.t[rt];
                const floatx4 c = tile_dot(tr.lo, o.Xf);
                bad |= tr.hi.x | tr.hi.y;
                const float d = f16_bits_to_f32(tr.sc & 0xffffu);
                const float z = f16_bits_to_f32(tr.sc >> 16);
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    acc[rt][i] = __builtin_fmaf(d, __builtin_fmaf(c[i], 16384.0f, -__builtin_fmaf(z, o.ev[i], o.sv[i])), acc[rt][i]);
            }
        }
    };
    auto compute = [&](const Slot& s, int j) {
        StepOperands o;
        prepare(o, s, j);
        compute_part(o, s, std::integral_constant<int, 0>{}, std::integral_constant<int, RT>{});
    };
    // One step of the pipeline: loads of step jn into `in`, arithmetic of step j from `cur`.  With many row
    // tiles the step runs in two halves (loads of the first tiles, arithmetic of the first tiles, then the
    // rest), so that the registers of the tiles already consumed carry the second half of the loads: the
    // two ring slots are never live in full at the same time.
    constexpr bool kHalves = RT >= 5;
    constexpr int RH = kHalves ? (RT + 1) / 2 : RT;
    auto step = [&](Slot& in, int jn, const Slot& cur, int j) {
        if constexpr (!kHalves) {
            issue(in, jn);
            compute(cur, j);
        } else {
            StepOperands o;
            issue_part(in, jn, std::integral_constant<int, 0>{}, std::integral_constant<int, RH>{});
            prepare(o, cur, j);
            compute_part(o, cur, std::integral_constant<int, 0>{}, std::integral_constant<int, RH>{});
            __builtin_amdgcn_sched_barrier(0);
            issue_part(in, jn, std::integral_constant<int, RH>{}, std::integral_constant<int, RT>{});
            compute_part(o, cur, std::integral_constant<int, RH>{}, std::integral_constant<int, RT>{});
        }
    };

    // ---- activations of this wavefront's blocks first (kFused), then the first D steps of tiles
    // (straight-line like the tile pipeline: slots past the wavefront's list re-read block 0 and are
    // rotated like the others; the host picks the smallest NBX that holds the list, because a load
    // costs address-unit time even when it hits)
    u32x2 xraw[kFused ? NBX * MP : 1];
    if constexpr (kFused) {
#pragma unroll
        for (int j = 0; j < NBX; ++j) {
            const int b = j < nb ? wave + j * W : 0;
#pragma unroll
            for (int m = 0; m < MP; ++m) {
                const int mr = m < a.M ? m : 0;
                xraw[j * MP + m] = *reinterpret_cast<const u32x2*>(a.X + (size_t)mr * a.ldx + (size_t)b * kBlock + 16 * r16 + 4 * g);
            }
        }
    }
    if constexpr (kFused) {
        // The rotations are interleaved with the first D steps of tile loads: a wavefront that issues
        // loads spends most of that time waiting for the address unit, and the rotation (a chain of
        // dependent matrix, convert and LDS instructions) fills those waits instead of following them.
        HadamardOperand H;
        H.init(lane);
        auto rotate_slot = [&](int j) {
#pragma unroll
            for (int m = 0; m < MP; ++m) {
                u32x2 raw = xraw[j * MP + m];
                if (m >= a.M) raw = u32x2{0u, 0u};
                const float s = rotate_to_lds<MP, !kMfmaSum>(raw, H, lane, m, xs + (size_t)j * MP * 256);
                // lane 0 holds x[0..3] of the chunk: E = 16 x_0
                const float e = 16.0f * (float)__builtin_bit_cast(_Float16, (uint16_t)(raw.x & 0xffffu));
                if constexpr (kMfmaSum) {
                    // no branch between the rotations of a slot: the other lanes write to a spare word each
                    float* dst = lane == 0 ? &se[j * MP + m] : &spare[lane];
                    *dst = e;
                } else if (lane == 0) {
                    ss[j * MP + m] = s;
                    se[j * MP + m] = e;
                }
            }
        };
#pragma unroll
        for (int d = 0; d < (D > NBX ? D : NBX); ++d) {
            if (d < D) issue(ring[d], d);
            __builtin_amdgcn_sched_barrier(0);
            if (d < NBX && d < nb) rotate_slot(d);  // (slots past the list hold block 0 again: nothing to rotate)
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
#pragma unroll
        for (int d = 0; d < D; ++d) issue(ring[d], d);
    }

    if (kFused && NBX <= 4 && D <= NBX && nb == NBX) {
        // The wavefront's list fills its slots exactly (K = 2048 NBX: 4096, 8192): a fixed schedule with
        // no stand-in loads behind the last step.
#pragma unroll
        for (int j = 0; j < NBX; ++j) {
            if (j + D < NBX) step(ring[(j + D) % NB], j + D, ring[j % NB], j);
            else compute(ring[j % NB], j);
        }
    } else {
        // ---- steady state: NB steps per trip, every prefetch is a live step
        int bi = 0;
        for (; bi + NB + D <= nb; bi += NB) {
#pragma unroll
            for (int k = 0; k < NB; ++k) {
                step(ring[(k + D) % NB], bi + k + D, ring[k], bi + k);
            }
        }
        // ---- tail: fewer than NB + D steps left
#pragma unroll
        for (int k = 0; k < NB + D - 1; ++k) {
            if (bi + k >= nb) break;  // straight line up to the exit: no merge point between steps
            step(ring[(k + D) % NB], bi + k + D, ring[k % NB], bi + k);
        }
    }

    // ---- add the W partial sums of every output, store Y.  red[wave][rt][m][r]; slot_out says where
    // the 16 outputs of a slot go.  (red overlaps nothing a wavefront still reads -- the rotated
    // activations and their sums lie in front of it -- so one barrier, behind the writes, is enough)
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (4 * g + i < MP) red[((wave * RT + rt) * MP + 4 * g + i) * 16 + r16] = acc[rt][i];
    __syncthreads();
    for (int o = threadIdx.x; o < RT * 16 * MP; o += W * 64) {
        const int rr = o % (RT * 16), m = o / (RT * 16);  // rr = rt*16 + r: consecutive threads, consecutive n
        const int rt = rr >> 4, r = rr & 15;
        const SlotOut so = slot_out[rt];
        if (r < so.rows && m < a.M) {
            float sum = 0.f;
#pragma unroll
            for (int wv = 0; wv < W; ++wv) sum += red[((wv * RT + rt) * MP + m) * 16 + r];
            const int64_t n = so.n0 + r;
            if (a.y_f16) reinterpret_cast<_Float16*>(so.Y)[m * so.ldy + n] = (_Float16)sum;
            else reinterpret_cast<float*>(so.Y)[m * so.ldy + n] = sum;
        }
    }
    if (a.flags != nullptr && bad != 0u) atomicOr(a.flags, kFlagBadCode);
}

template <int MP, int RT, int D, int NBX, bool kGrouped>
static int launch_kernel(const GemvArgs& a, int grid, hipStream_t stream) {
    auto kern = gemv_kernel<MP, RT, D, NBX, kGrouped>;
    static std::atomic<bool> lds_limit_raised{false};  // once per instantiation: allow up to the 160 KB of a CU
    if (!lds_limit_raised) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) return -6;
        lds_limit_raised = true;
    }
    const size_t lds = (size_t)kGemvWaves * NBX * MP * (512 + 8) + (size_t)kGemvWaves * RT * MP * 16 * 4 + (size_t)RT * 32 + (size_t)kGemvWaves * 256;
    const LaunchTiming tm = take_launch_timing();
    if (tm.start != nullptr) hipExtLaunchKernelGGL(kern, dim3(grid), dim3(kGemvWaves * 64), lds, stream, tm.start, tm.stop, 0, a);
    else hipLaunchKernelGGL(kern, dim3(grid), dim3(kGemvWaves * 64), lds, stream, a);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

template <int MP, int RT, int D, int NBX>
static int launch_one(const GemvArgs& a, int grid, hipStream_t stream) {
    if (a.t[1].v_begin != 0x7fffffff) return launch_kernel<MP, RT, D, NBX, true>(a, grid, stream);
    return launch_kernel<MP, RT, D, NBX, false>(a, grid, stream);
}

// Prefetch depth the register file allows for RT row tiles per workgroup (the direct path keeps the
// x~ fragments in the ring too, MP = 4 rotates four rows per block).
template <int MP, bool kFused>
constexpr int max_depth(int rt) {
    if (kFused) return rt <= 2 ? 4 : (rt == 3 || (rt == 4 && MP <= 2)) ? 2 : 1;
    return rt == 1 ? (MP >= 8 ? 2 : 4) : rt <= 3 ? 2 : 1;  // (8 rows and more, depth 4: the ring would spill)
}

// Smallest of 2, 4, 8, 16 that holds nb_max blocks per wavefront (fused path); 0 = direct.
template <int MP, int RT, int D, bool kFused>
static int launch_nbx(const GemvArgs& a, int grid, int nb_max, hipStream_t stream) {
    if constexpr (D > max_depth<MP, kFused>(RT)) {
        return -6;
    } else if constexpr (!kFused) {
        return launch_one<MP, RT, D, 0>(a, grid, stream);
    } else {
        // D <= blocks of the least busy wavefront <= nb_max <= NBX: deeper combinations cannot occur
        if (nb_max <= 2) {
            if constexpr (D <= 2) return launch_one<MP, RT, D, 2>(a, grid, stream);
        } else if (nb_max <= 4) {
            if constexpr (4 * MP <= fused_max_blocks(MP) && D <= 4) return launch_one<MP, RT, D, 4>(a, grid, stream);
        } else if (nb_max <= 8) {
            if constexpr (8 * MP <= fused_max_blocks(MP) && D == max_depth<MP, kFused>(RT)) return launch_one<MP, RT, D, 8>(a, grid, stream);
        } else if (nb_max <= 16) {
            if constexpr (16 * MP <= fused_max_blocks(MP) && D == max_depth<MP, kFused>(RT)) return launch_one<MP, RT, D, 16>(a, grid, stream);
        }
        return -6;  // no instantiation holds this many blocks per wavefront: gemv_can_fuse() excludes it
    }
}

template <int MP, int RT, bool kFused>
static int launch_depth(const GemvArgs& a, int grid, int nb_min, int nb_max, hipStream_t stream) {
    // about 8 tiles in flight per wavefront, never deeper than the shortest wavefront's list of blocks
    // (deeper would only add stand-in loads)
    int d = max_depth<MP, kFused>(RT);
    while (d > 1 && d > nb_min) d >>= 1;
    switch (d) {
        case 4: return launch_nbx<MP, RT, 4, kFused>(a, grid, nb_max, stream);
        case 2: return launch_nbx<MP, RT, 2, kFused>(a, grid, nb_max, stream);
        default: return launch_nbx<MP, RT, 1, kFused>(a, grid, nb_max, stream);
    }
}

template <int MP, bool kFused>
static int launch_shape(const GemvArgs& a, int grid, int rt, int nb_min, int nb_max, hipStream_t stream) {
    switch (rt) {
        case 1: return launch_depth<MP, 1, kFused>(a, grid, nb_min, nb_max, stream);
        case 2: return launch_depth<MP, 2, kFused>(a, grid, nb_min, nb_max, stream);
        case 3: return launch_depth<MP, 3, kFused>(a, grid, nb_min, nb_max, stream);
        case 4: return launch_depth<MP, 4, kFused>(a, grid, nb_min, nb_max, stream);
        case 5: return launch_depth<MP, 5, kFused>(a, grid, nb_min, nb_max, stream);
        case 6: return launch_depth<MP, 6, kFused>(a, grid, nb_min, nb_max, stream);
        default: return launch_depth<MP, 7, kFused>(a, grid, nb_min, nb_max, stream);
    }
}

int launch_gemv(const GemvWeight* w, int count, int64_t K, const _Float16* X, int64_t ldx, const float* S, int64_t M, int MP, bool fused,
                int y_f16, uint32_t* flags, hipStream_t stream) {
    if (count < 1 || count > kGemvMaxGroup) return -2;
    GemvArgs a;
    a.X = X; a.S = S; a.flags = flags; a.ldx = ldx; a.KB = (int)(K / kBlock); a.M = (int)M; a.y_f16 = y_f16;
    // One workgroup per CU if that leaves at most kGemvMaxRT row tiles each, else more workgroups.
    // (The kernel's registers allow one workgroup per CU at a time, so a grid just above the CU count
    // would run a nearly empty second round.)  The row tiles of all tensors form one list, split
    // evenly: every workgroup gets rt or rt-1 of them.
    int64_t nt_total = 0;
    for (int i = 0; i < kGemvMaxGroup; ++i) {
        GemvTensor& t = a.t[i];
        if (i < count) {
            t.codes = w[i].codes; t.scales = w[i].scales; t.Y = w[i].Y; t.N = w[i].N; t.ldy = w[i].ldy;
            if (nt_total > 0x7fffffff) return -2;
            t.v_begin = (int)nt_total;
            nt_total += (w[i].N + 15) / 16;
        } else {
            t = a.t[0];
            t.v_begin = 0x7fffffff;
        }
        t.pad_ = 0;
    }
    if (nt_total >= 0x7fffffff) return -2;
    const int nb_min = a.KB / kGemvWaves, nb_max = (a.KB + kGemvWaves - 1) / kGemvWaves;
    // row tiles per workgroup, at most: the register ring's limit, and with many fused rows what the LDS
    // leaves next to the rotated activations (8 NBX MP 520 bytes; 8 MP 64 bytes of partial sums per tile)
    int max_rt = kGemvMaxRT;
    if (fused) {
        const int nbx = nb_max <= 2 ? 2 : nb_max <= 4 ? 4 : nb_max <= 8 ? 8 : 16;
        const int64_t room = 160 * 1024 - 4096 - (int64_t)kGemvWaves * nbx * MP * (512 + 8);
        const int64_t fit = room / ((int64_t)kGemvWaves * MP * 64 + 32);
        if (fit < 1) return -2;
        if (fit < max_rt) max_rt = (int)fit;
    }
    int64_t grid64 = nt_total < cu_count() ? nt_total : cu_count();
    if ((nt_total + grid64 - 1) / grid64 > max_rt) grid64 = (nt_total + max_rt - 1) / max_rt;
    const int grid = (int)grid64;
    const int rt = (int)((nt_total + grid - 1) / grid);
    a.nt_q = (int)(nt_total / grid);
    a.nt_r = (int)(nt_total % grid);
    switch (MP) {
        case 8: return launch_shape<8, false>(a, grid, rt, nb_min, nb_max, stream);
        case 16: return launch_shape<16, false>(a, grid, rt, nb_min, nb_max, stream);
    }
    return -2;
}

}  // namespace rows

int launch_gemv_rows(const GemvWeight* w, int count, int64_t K, const _Float16* Xt, const float* S, int64_t M, int MP, int y_f16,
                     uint32_t* flags, hipStream_t stream) {
    return rows::launch_gemv(w, count, K, Xt, 0, S, M, MP, false, y_f16, flags, stream);
}

}  // namespace itq3s
