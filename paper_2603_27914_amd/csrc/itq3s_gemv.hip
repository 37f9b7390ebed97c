// Streaming matmul for M <= 16 activation rows (the decode path, Sec. 5.4).  The description below is
// the kernel for M <= 4, which rotates the activations itself; the variant for 5..16 rows, which
// takes them rotated from a launch in front, is described at the kernel template.
//
//   Y[m][n] = sum_b d[n,b] * ( sum_j c[n,b,j] x~[m,b,j]  -  S[m,b]  -  z[n,b] * E[m,b] )
//
// with c = q+1 the stored code, x~ = H x the rotated activation chunk rounded to fp16 (H is
// symmetric and its own inverse, Sec. 2.3: <H v, x> = <v, H x>, so the rotation is applied to the
// activations and the packed weights are consumed as stored), S[m,b] = sum_j x~[m,b,j] over those
// rounded values (it cancels the +1 of the codes exactly) and E[m,b] = 16 x[m, 256 b], the exact
// value of the same sum before rounding (H 1 = 16 e_0): the zero-point term is formed from the
// activations themselves, so the rounding of x~ is not multiplied by z.  The packed weights are read
// exactly once -- one 16-byte + one 8-byte + one 4-byte (scale) load per lane and tile -- and nothing
// dequantized is written anywhere.
//
// Contraction: v_mfma_f32_16x16x32_f16 with the activations as the A operand (rows = m) and 16
// weight rows of a tile as the B operand (columns = n), so that every accumulator of a lane belongs
// to the lane's own weight row and needs only that row's scale.  A code c in {0,1,2} placed in bits
// 11:10 of a half is the number c * 2^-14, so two codes that sit 16 bits apart in a low-plane word
// become a half2 with one shift and one mask; the factor 2^14 is applied together with d.
//
// Work split: workgroup g (8 wavefronts) owns RT or RT-1 consecutive 16-row tiles of the launch and
// all of K; wavefront w takes blocks w, w+8, ...  A step of a wavefront is one block against the
// workgroup's row tiles: the tile loads of the next step are in flight (two register buffers) while
// the wavefront rotates the 256 activations of its current block on the matrix cores, parks them in
// its private 512 M bytes of LDS in operand order, and multiplies.  No wavefront waits for another
// before the cross-wavefront sum at the end.  Every load goes through a buffer descriptor: a row
// tile the workgroup does not have gets an empty descriptor (its loads return zeros without touching
// memory), so the step is branch-free.  The kernel needs 86 to 128 registers, which leaves room for
// two workgroups per compute unit: one workgroup's start-up and final sum overlap the other's
// streaming.
#include <hip/hip_ext.h>

#include "itq3s_dev.h"
#include <atomic>
#include <type_traits>

#include "itq3s_kernels.h"

namespace itq3s {

constexpr int kGemvWaves = 8;      // wavefronts per workgroup
constexpr int kGemvMaxRT = 3;      // row tiles per workgroup, at most (7 registers per tile and buffer; four would cost the second workgroup per compute unit)
constexpr int kRawBuffer = 0x00027000;  // buffer descriptor word 3: raw buffer of 32-bit elements
constexpr int kLoadNT = 2;         // cache policy of the weight loads: nontemporal (read once)

static thread_local LaunchTiming g_timing;  // armed and taken on the calling thread
void set_launch_timing(hipEvent_t start, hipEvent_t stop) { g_timing.start = start; g_timing.stop = stop; }
LaunchTiming take_launch_timing() {
    const LaunchTiming t = g_timing;
    g_timing = LaunchTiming{};
    return t;
}

// One launch serves up to kGemvMaxGroup weight tensors that share K and the activations (the
// projections of one layer that read the same input).  Their 16-row tiles are numbered as one list,
// tensor after tensor, and split evenly over the workgroups; a workgroup's tiles may belong to two
// tensors.
struct GemvTensor {
    const uint32_t* codes;
    const uint32_t* scales;
    const uint32_t* subscales;  // the 116-byte variant's sub-scale array, or null
    void* Y;
    int64_t N, ldy;
    int v_begin;  // position of this tensor's first row tile in the list (0x7fffffff for unused entries)
    int pad_;
};

struct GemvArgs {
    GemvTensor t[kGemvMaxGroup];
    const _Float16* X;  // activations [M][ldx]; kRotated: x~ in operand order with MP columns (from the rotation launch)
    const float* S;     // kRotated: [2][KB][MP] sums of the rounded x~ per block and row, then 16 x[m][256 b]
    uint32_t* flags;
    int64_t ldx;
    int KB, M, y_f16;
    int nt_q, nt_r;  // row tiles per workgroup: the first nt_r workgroups own nt_q + 1, the others nt_q
};

struct TileRegs {
    u32x4 lo;
    u32x2 hi;
    uint32_t sc;
    uint32_t ss;  // (sub-block variant) the lane's two sub-scales
};

__device__ __forceinline__ half8 as_half8(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
    u32x4 u = {a, b, c, d};
    return __builtin_bit_cast(half8, u);
}

// The 256-point transform on the matrix cores.  With the chunk written as a 16 x 16 matrix
// X[a][b] = x[16a + b], the Sylvester construction gives H_256 = H_16 (x) H_16, i.e.
//     (H x)[16a' + b'] = (H_16 X H_16)[a'][b'] / 16        (H_16 with entries +-1).
// Two 16x16x16 products do it: T = X (H_16/4) (fp16 inputs, exact products, fp32 sums; the factor
// keeps |T| <= 4 max|x|), then H_16 T with T split into two halves (T = T_hi + T_lo keeps 22
// bits), then the remaining factor 1/4.  The accumulator layout of the first product (lane = column
// b', four rows a per lane) is exactly the B-operand layout of the second, so nothing moves between
// lanes.  A lane holds x[16 (l%16) + 4 (l/16) + 0..3] on entry and element e = 64 (l/16) + 16 r + l%16,
// r = 0..3, of the result.
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
// index ((t*4 + g)*MP + m)*8 + i).  Returns false if a rotated value (or the intermediate T, which
// then turns the result into NaN) leaves the fp16 range.
template <int MP>
__device__ __forceinline__ bool rotate_to_lds(u32x2 raw, const HadamardOperand& H, int lane, int m, _Float16* dst) {
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
    bool ok = true;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        r[i] = (_Float16)(U[i] * 0.25f);
        ok = ok && __builtin_fabsf(U[i]) <= 4.0f * 65504.0f;  // (false for NaN as well)
    }
    // element e = 64g + 16w + slot (w = r, slot = l%16): quarter g, low-plane word w, code slot `slot`;
    // MFMA step t = 2w + ((slot&7)>>2), position i = 2(slot&3) + (slot>>3)
    const int g = lane >> 4, slot = lane & 15;
    const int tb = (slot & 7) >> 2, i0 = 2 * (slot & 3) + (slot >> 3);
#pragma unroll
    for (int w = 0; w < 4; ++w) dst[(((2 * w + tb) * 4 + g) * MP + m) * 8 + i0] = r[w];
    return ok;
}

// kGrouped: the launch serves several tensors (a single-tensor launch skips the lookup and the
// fetch of the unused descriptors, which are on the way to the first load).
// NBC > 0: every wavefront has exactly NBC blocks (K = 2048 NBC): the pipeline is straight-line code,
// which the compiler fits into 57..92 registers instead of 86..126 -- a third workgroup per compute unit.
// kSub: the sub-block-scale variant of the format (Sec. 4.1: 116 bytes per block), one tensor per launch:
//   Y[m][n] = sum_b d ( sum_j s[n,b,j/32] (c-1)[n,b,j] x~[m,b,j]  -  z E[m,b] ).
// A lane's 64 codes belong to two sub-blocks (low-plane words 0,1 and 2,3), whose scales are the two
// halves of one more word per lane and tile.  The operand is the signed digit times the sub-scale:
// (c 2^-14) (16 s) - s 2^-10 = (c-1) s 2^-10, exact in fp16 for 2^-4 <= s <= 4094 (the quantizer's
// sub-scales lie below 3; smaller ones lose low bits of a contribution that is small anyway), so no
// block sum S is needed.
// kRotated (5..16 rows, MP = 8 or 16; either format): the activations arrive rotated, in operand order, from a launch
// of their own (rotating 8 or 16 rows per block inside every workgroup would cost more than the
// contraction); a wavefront loads the eight fragments and the two sums of its next block straight into
// registers right behind the arithmetic of the current one, in front of the next tile loads, so that
// the in-order load counter never makes it wait for those.
// NSG = 2 (kRotated only): the workgroup owns 2 RT row tiles; a wavefront multiplies the fragments of a
// block with the first RT tiles, then with the other RT (two pipeline steps per block), so that every
// fragment fetched -- the bulk of what a workgroup pulls through its L1 with 16 rows -- serves twice
// the weights, and its latency is met once per two steps.
template <int MP, int RT, bool kGrouped, int NBC, bool kSub = false, bool kRotated = false, int NSG = 1>
// (launch bounds: the second figure is a lower bound on wavefronts per SIMD: 4 = two workgroups per
// compute unit = at most 128 registers, which every instantiation of the general pipeline meets
// without scratch; the straight-line kernels use 57..92 registers on their own)
__global__ __launch_bounds__(kGemvWaves * 64, NBC > 0 ? 3 : 4) void gemv_kernel(const GemvArgs a) {
    static_assert(!kRotated || (NBC == 0 && MP >= 8), "rotated activations: general pipeline");
    static_assert(kRotated || MP <= 4, "in-kernel rotation: at most four rows");
    static_assert(NSG == 1 || (NSG == 2 && kRotated), "row sub-groups: with rotated activations only");
    constexpr int RTW = RT * NSG;  // row tiles of the workgroup
    constexpr int W = kGemvWaves;
    extern __shared__ __align__(16) unsigned char smem[];
    const int KB = a.KB;
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));  // wave-uniform, in an SGPR
    const int g = lane >> 4, r16 = lane & 15, mm = r16 & (MP - 1);
    const int wg = (int)blockIdx.x;
    const int nt_begin = wg * a.nt_q + (wg < a.nt_r ? wg : a.nt_r);
    const int cnt = a.nt_q + (wg < a.nt_r ? 1 : 0);
    struct SlotOut {   // where the 16 outputs of a slot go (table in LDS, read back in the epilogue)
        void* Y;
        int64_t ldy;
        int64_t n0;    // first row of the tile inside its tensor
        int64_t rows;  // rows of that tensor from n0 on that exist (<= 0: slot unused)
    };
    // LDS: per wavefront MP*512 bytes of x~ (in-kernel rotation only) | red: W*RTW*MP*16 floats | slot_out[RTW]
    constexpr size_t kXsBytes = kRotated ? 0 : (size_t)W * MP * 512;
    _Float16* const xs = reinterpret_cast<_Float16*>(smem) + (size_t)wave * MP * 256;
    float* const red = reinterpret_cast<float*>(smem + kXsBytes);
    SlotOut* const slot_out = reinterpret_cast<SlotOut*>(smem + kXsBytes + (size_t)W * RTW * MP * 16 * 4);

    // Per slot: descriptors over the K range of the tile row in codes / scales (scalar selects; all
    // tensor entries come with the first argument fetch).
    __amdgpu_buffer_rsrc_t crs[RTW], srs[RTW], urs[kSub ? RTW : 1];
    void* so_y[RTW];  // the output table's entries: written behind the first loads, they are not needed before the end
    int64_t so_ldy[RTW], so_n0[RTW], so_rows[RTW];
    // grouped: the tensor of a slot is found from the three list positions alone, and its entry is then
    // fetched from the argument block by index (one scalar load per slot, all in flight together) --
    // selecting every field among four entries took 340 scalar instructions and nine dependent fetches
    // in front of the first weight load
    [[maybe_unused]] const auto* const kargs = (const __attribute__((address_space(4))) GemvArgs*)__builtin_amdgcn_kernarg_segment_ptr();
    [[maybe_unused]] const int vb1 = a.t[1].v_begin, vb2 = a.t[2].v_begin, vb3 = a.t[3].v_begin;
#pragma unroll
    for (int rt = 0; rt < RTW; ++rt) {
        const uint32_t* t_codes = a.t[0].codes;
        const uint32_t* t_scales = a.t[0].scales;
        void* t_y = a.t[0].Y;
        int64_t t_n = a.t[0].N, t_ldy = a.t[0].ldy;
        int t_begin = 0;
        if constexpr (kGrouped) {
            const int tile = nt_begin + rt;
            const int ti = (tile >= vb1 ? 1 : 0) + (tile >= vb2 ? 1 : 0) + (tile >= vb3 ? 1 : 0);  // list positions ascend; unused entries hold INT_MAX
            t_codes = kargs->t[ti].codes;
            t_scales = kargs->t[ti].scales;
            t_y = kargs->t[ti].Y;
            t_n = kargs->t[ti].N;
            t_ldy = kargs->t[ti].ldy;
            t_begin = kargs->t[ti].v_begin;
        }
        const bool have = rt < cnt;
        const int64_t local = nt_begin + rt - t_begin;
        const int64_t first = have ? local * KB : 0;
        crs[rt] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(t_codes + first * kTileWords), 0, have ? KB * 1536 : 0, kRawBuffer);
        srs[rt] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(t_scales + first * kTileRows), 0, have ? KB * 64 : 0, kRawBuffer);
        if constexpr (kSub) urs[rt] = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(a.t[0].subscales + first * 64), 0, have ? KB * 256 : 0, kRawBuffer);
        so_y[rt] = t_y;
        so_ldy[rt] = t_ldy;
        so_n0[rt] = local * 16;
        so_rows[rt] = have ? t_n - local * 16 : 0;
    }
    // activations: rows beyond M read as zeros (offset outside the descriptor's range)
    const __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<_Float16*>(a.X), 0, kRotated ? KB * MP * 512 : (int)(((int64_t)(a.M - 1) * a.ldx + (int64_t)KB * 256) * 2), kRawBuffer);
    const __amdgpu_buffer_rsrc_t sumrs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.S), 0, kRotated ? 2 * KB * MP * 4 : 0, kRawBuffer);
    const int nb = KB > wave ? (KB - wave + W - 1) / W : 0;  // blocks of this wavefront: b = wave + j*W

    constexpr uint32_t kOutside = 0x80000000u;  // an offset no descriptor here covers
    const uint32_t none = nb > 0 ? 0u : kOutside;  // a wavefront without blocks (K < 2048) loads nothing
    const uint32_t off_lo = lane * 16 + none, off_hi = lane * 8 + 1024 + none, off_sc = r16 * 4 + none, off_ss = lane * 4 + none;
    uint32_t off_x[kRotated ? 1 : MP];
    if constexpr (!kRotated) {
#pragma unroll
        for (int m = 0; m < MP; ++m) off_x[m] = m < a.M ? ((uint32_t)(m * a.ldx * 2) + (16 * r16 + 4 * g) * 2) | none : kOutside;
    }
    // rotated activations: fragment t of the block for lane (row mm, quarter g) at ((t*4 + g)*MP + mm)*16 bytes
    const uint32_t off_xf = (uint32_t)((g * MP + mm) * 16) + none, off_sum = (uint32_t)(((4 * g) & (MP - 1)) * 4) + none;
    half8 xf[kRotated ? 8 : 1];
    floatx4 sv_r = {0.f, 0.f, 0.f, 0.f}, ev_r = {0.f, 0.f, 0.f, 0.f};
    auto issue_x = [&](int j) {  // fragments and sums of step j (kRotated)
        const int b = nb > 0 ? wave + j * W : 0;
#pragma unroll
        for (int t = 0; t < 8; ++t)
            xf[t] = __builtin_bit_cast(half8, __builtin_amdgcn_raw_buffer_load_b128(xrs, off_xf + (uint32_t)(t * 4 * MP * 16), b * (MP * 512), 0));
        sv_r = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(sumrs, off_sum, b * (MP * 4), 0));
        ev_r = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(sumrs, off_sum, (KB + b) * (MP * 4), 0));
    };

    floatx4 acc[RTW];
#pragma unroll
    for (int rt = 0; rt < RTW; ++rt) acc[rt] = floatx4{0.f, 0.f, 0.f, 0.f};
    uint32_t bad = 0;
    bool in_range = true;

    struct Slot {
        TileRegs t[RT];
        u32x2 xr[kRotated ? 1 : MP];
    };
    Slot ring[2];

    // loads of step j: the wavefront's activations of block wave + j*W, then that block of every row tile
    // (of sub-group SG of the row tiles)
    auto issue_sg = [&](Slot& s, int j, auto sgc) {
        constexpr int SG = decltype(sgc)::value;
        const int b = nb > 0 ? wave + j * W : 0;
        if constexpr (!kRotated) {
#pragma unroll
            for (int m = 0; m < MP; ++m) s.xr[m] = __builtin_amdgcn_raw_buffer_load_b64(xrs, off_x[m], b * 512, 0);
        }
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            s.t[rt].lo = __builtin_amdgcn_raw_buffer_load_b128(crs[SG * RT + rt], off_lo, b * 1536, kLoadNT);
            s.t[rt].hi = __builtin_amdgcn_raw_buffer_load_b64(crs[SG * RT + rt], off_hi, b * 1536, kLoadNT);
            s.t[rt].sc = __builtin_amdgcn_raw_buffer_load_b32(srs[SG * RT + rt], off_sc, b * 64, kLoadNT);
            if constexpr (kSub) s.t[rt].ss = __builtin_amdgcn_raw_buffer_load_b32(urs[SG * RT + rt], off_ss, b * 256, kLoadNT);
        }
    };
    auto issue = [&](Slot& s, int j) { issue_sg(s, j, std::integral_constant<int, 0>{}); };

    HadamardOperand H;
    H.init(lane);
    const half8 ones = as_half8(0x04000400u, 0x04000400u, 0x04000400u, 0x04000400u);  // 2^-14 each

    auto compute_sg = [&](const Slot& s, auto sgc) {
        constexpr int SG = decltype(sgc)::value;
        float ev[4];
        if constexpr (kRotated) {
#pragma unroll
            for (int i = 0; i < 4; ++i) ev[i] = ev_r[i];
        } else {
#pragma unroll
            for (int m = 0; m < MP; ++m) in_range = rotate_to_lds<MP>(s.xr[m], H, lane, m, xs) && in_range;
            // lane 0 holds x[0..3] of the chunk: E = 16 x_0 (rows m = 4g + i of the accumulators are row i & (MP-1) for M <= 4)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t w0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)s.xr[i & (MP - 1)].x);
                ev[i] = 16.0f * f16_bits_to_f32(w0 & 0xffffu);
            }
        }
        // the block sums S come from the matrix cores as well: the same fragments against an operand of ones
        floatx4 sacc = {0.f, 0.f, 0.f, 0.f};
        floatx4 c[RT];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) c[rt] = floatx4{0.f, 0.f, 0.f, 0.f};
        half8 sub_mul[kSub ? RT : 1][2], sub_add[kSub ? RT : 1][2];  // (sub-block variant) 16 s and -s 2^-10 of the lane's two sub-blocks
        if constexpr (kSub) {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                const half2v s2 = __builtin_bit_cast(half2v, s.t[rt].ss);
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const _Float16 m = s2[h] * (_Float16)16.0f, n = s2[h] * (_Float16)(-0.0009765625f);
                    sub_mul[rt][h] = half8{m, m, m, m, m, m, m, m};
                    sub_add[rt][h] = half8{n, n, n, n, n, n, n, n};
                }
            }
        }
        constexpr uint32_t kMask = 0x0C000C00u;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            half8 Xf;
            if constexpr (kRotated) Xf = xf[t];
            else Xf = *reinterpret_cast<const half8*>(xs + ((t * 4 + g) * MP + mm) * 8);
            if constexpr (!kSub && !kRotated) sacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(Xf, ones, sacc, 0, 0, 0);
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                const uint32_t wds[4] = {s.t[rt].lo.x, s.t[rt].lo.y, s.t[rt].lo.z, s.t[rt].lo.w};
                const uint32_t v = wds[t >> 1];
                // slots j and j+8 of the word -> bits 11:10 and 27:26
                half8 op = (t & 1) == 0 ? as_half8((v << 10) & kMask, (v << 8) & kMask, (v << 6) & kMask, (v << 4) & kMask)
                                        : as_half8((v << 2) & kMask, v & kMask, (v >> 2) & kMask, (v >> 4) & kMask);
                if constexpr (kSub) op = __builtin_elementwise_fma(op, sub_mul[rt][t >> 2], sub_add[rt][t >> 2]);  // words 0,1 | 2,3
                c[rt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(Xf, op, c[rt], 0, 0, 0);
            }
        }
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            bad |= s.t[rt].hi.x | s.t[rt].hi.y;
            const float d = f16_bits_to_f32(s.t[rt].sc & 0xffffu);
            const float z = f16_bits_to_f32(s.t[rt].sc >> 16);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                acc[SG * RT + rt][i] = kSub       ? __builtin_fmaf(d, __builtin_fmaf(c[rt][i], 1024.0f, -z * ev[i]), acc[SG * RT + rt][i])
                                       : kRotated ? __builtin_fmaf(d, __builtin_fmaf(c[rt][i], 16384.0f, -__builtin_fmaf(z, ev[i], sv_r[i])), acc[SG * RT + rt][i])
                                                  : __builtin_fmaf(d, __builtin_fmaf(c[rt][i] - sacc[i], 16384.0f, -z * ev[i]), acc[SG * RT + rt][i]);
        }
    };
    auto compute = [&](const Slot& s) { compute_sg(s, std::integral_constant<int, 0>{}); };

    // ---- pipeline, one step ahead; every load issued belongs to a real step (the scheduling
    // barriers keep the loads in front of the arithmetic they overlap with)
    issue(ring[0], 0);
    if constexpr (kRotated) issue_x(0);
    __builtin_amdgcn_sched_barrier(0);
    if (threadIdx.x == 0) {
#pragma unroll
        for (int rt = 0; rt < RTW; ++rt) slot_out[rt] = SlotOut{so_y[rt], so_ldy[rt], so_n0[rt], so_rows[rt]};
    }
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (NBC > 0) {
#pragma unroll
        for (int q = 0; q < NBC; ++q) {
            if (q + 1 < NBC) issue(ring[(q + 1) & 1], q + 1);
            __builtin_amdgcn_sched_barrier(0);
            compute(ring[q & 1]);
            __builtin_amdgcn_sched_barrier(0);
        }
    } else if constexpr (NSG == 2) {
        // two steps per block: ring[0] carries the first RT row tiles of a block, ring[1] the others
        constexpr std::integral_constant<int, 0> sg0{};
        constexpr std::integral_constant<int, 1> sg1{};
        int j = 0;
        for (; j + 1 < nb; ++j) {
            issue_sg(ring[1], j, sg1);
            __builtin_amdgcn_sched_barrier(0);
            compute_sg(ring[0], sg0);
            __builtin_amdgcn_sched_barrier(0);
            issue_sg(ring[0], j + 1, sg0);
            __builtin_amdgcn_sched_barrier(0);
            compute_sg(ring[1], sg1);
            __builtin_amdgcn_sched_barrier(0);
            issue_x(j + 1);
        }
        if (nb > 0) {
            issue_sg(ring[1], j, sg1);
            __builtin_amdgcn_sched_barrier(0);
            compute_sg(ring[0], sg0);
            __builtin_amdgcn_sched_barrier(0);
            compute_sg(ring[1], sg1);
        }
    } else {
        int j = 0;
        for (; j + 2 < nb; j += 2) {
            issue(ring[1], j + 1);
            __builtin_amdgcn_sched_barrier(0);
            compute(ring[0]);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (kRotated) issue_x(j + 1);
            issue(ring[0], j + 2);
            __builtin_amdgcn_sched_barrier(0);
            compute(ring[1]);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (kRotated) issue_x(j + 2);
        }
        if (j + 2 == nb) {
            issue(ring[1], j + 1);
            __builtin_amdgcn_sched_barrier(0);
            compute(ring[0]);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (kRotated) issue_x(j + 1);
            __builtin_amdgcn_sched_barrier(0);
            compute(ring[1]);
        } else if (j + 1 == nb) {
            compute(ring[0]);
        }
    }

    // ---- add the W partial sums of every output, store Y.  red[wave][rt][m][r]; slot_out says where
    // the 16 outputs of a slot go.
#pragma unroll
    for (int rt = 0; rt < RTW; ++rt)
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (4 * g + i < MP) red[((wave * RTW + rt) * MP + 4 * g + i) * 16 + r16] = acc[rt][i];
    __syncthreads();
    for (int o = threadIdx.x; o < RTW * 16 * MP; o += W * 64) {
        const int rr = o % (RTW * 16), m = o / (RTW * 16);  // rr = rt*16 + r: consecutive threads, consecutive n
        const int rt = rr >> 4, r = rr & 15;
        const SlotOut so = slot_out[rt];
        if (r < so.rows && m < a.M) {
            float sum = 0.f;
#pragma unroll
            for (int wv = 0; wv < W; ++wv) sum += red[((wv * RTW + rt) * MP + m) * 16 + r];
            const int64_t n = so.n0 + r;
            if (a.y_f16) reinterpret_cast<_Float16*>(so.Y)[m * so.ldy + n] = (_Float16)sum;
            else reinterpret_cast<float*>(so.Y)[m * so.ldy + n] = sum;
        }
    }
    if (a.flags != nullptr) {
        const uint32_t f = (bad != 0u ? kFlagBadCode : 0u) | (in_range ? 0u : kFlagActRange);
        if (f != 0u) atomicOr(a.flags, f);
    }
}

template <int MP, int RT, bool kGrouped, int NBC, bool kSub = false, bool kRotated = false, int NSG = 1>
static int launch_kernel(const GemvArgs& a, int grid, hipStream_t stream) {
    auto kern = gemv_kernel<MP, RT, kGrouped, NBC, kSub, kRotated, NSG>;
    const size_t lds = (kRotated ? 0 : (size_t)kGemvWaves * MP * 512) + (size_t)kGemvWaves * RT * NSG * MP * 16 * 4 + (size_t)RT * NSG * 32;
    const LaunchTiming tm = take_launch_timing();
    if (tm.start != nullptr) hipExtLaunchKernelGGL(kern, dim3(grid), dim3(kGemvWaves * 64), lds, stream, tm.start, tm.stop, 0, a);
    else hipLaunchKernelGGL(kern, dim3(grid), dim3(kGemvWaves * 64), lds, stream, a);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

template <int MP, int RT, int NBC>
static int launch_one(const GemvArgs& a, int grid, hipStream_t stream) {
    if (a.t[1].v_begin != 0x7fffffff) return launch_kernel<MP, RT, true, NBC>(a, grid, stream);
    return launch_kernel<MP, RT, false, NBC>(a, grid, stream);
}

template <int MP, int NBC>
static int launch_shape(const GemvArgs& a, int grid, int rt, hipStream_t stream) {
    switch (rt) {
        case 1: return launch_one<MP, 1, NBC>(a, grid, stream);
        case 2: return launch_one<MP, 2, NBC>(a, grid, stream);
        case 3: return launch_one<MP, 3, NBC>(a, grid, stream);
    }
    return -2;
}

template <int MP>
static int launch_blocks(const GemvArgs& a, int grid, int rt, hipStream_t stream) {
    if (a.t[0].subscales != nullptr) {  // the sub-block variant: one tensor, the general pipeline
        switch (rt) {
            case 1: return launch_kernel<MP, 1, false, 0, true>(a, grid, stream);
            case 2: return launch_kernel<MP, 2, false, 0, true>(a, grid, stream);
            case 3: return launch_kernel<MP, 3, false, 0, true>(a, grid, stream);
        }
        return -2;
    }
    if (a.KB == 8) return launch_shape<MP, 1>(a, grid, rt, stream);
    if (a.KB == 16) return launch_shape<MP, 2>(a, grid, rt, stream);
    return launch_shape<MP, 0>(a, grid, rt, stream);
}

int cu_count() {
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

// Fills the tensor list of a launch; returns the number of row tiles, or -1.
static int64_t fill_tensors(GemvArgs& a, const GemvWeight* w, int count) {
    int64_t nt_total = 0;
    for (int i = 0; i < kGemvMaxGroup; ++i) {
        GemvTensor& t = a.t[i];
        if (i < count) {
            t.codes = w[i].codes; t.scales = w[i].scales; t.subscales = w[i].subscales; t.Y = w[i].Y; t.N = w[i].N; t.ldy = w[i].ldy;
            if (t.subscales != nullptr && count != 1) return -1;
            if (nt_total > 0x7fffffff) return -1;
            t.v_begin = (int)nt_total;
            nt_total += (w[i].N + 15) / 16;
        } else {
            t = a.t[0];
            t.v_begin = 0x7fffffff;
        }
        t.pad_ = 0;
    }
    return nt_total < 0x7fffffff ? nt_total : -1;
}

int launch_gemv(const GemvWeight* w, int count, int64_t K, const _Float16* X, int64_t ldx, int64_t M, int y_f16, uint32_t* flags,
                hipStream_t stream) {
    if (count < 1 || count > kGemvMaxGroup || M < 1 || M > kGemvFusedMaxM) return -2;
    GemvArgs a;
    a.X = X; a.S = nullptr; a.flags = flags; a.ldx = ldx; a.KB = (int)(K / kBlock); a.M = (int)M; a.y_f16 = y_f16;
    const int64_t nt_total = fill_tensors(a, w, count);
    if (nt_total < 0) return -2;
    // Row tiles per workgroup (every workgroup rotates all of X for itself, so more tiles per workgroup
    // mean less of that; fewer mean more workgroups in flight).  Measured on the 7B and 70B shapes:
    //  - K = 2048 or 4096 (a wavefront walks one or two blocks; three or four workgroups fit a compute
    //    unit): the fewest tiles per workgroup that keep the grid within three workgroups per unit;
    //  - otherwise: as many tiles as keep one workgroup per compute unit busy, at most three.
    const int cus = cu_count();
    int64_t grid64;
    if ((a.KB == 8 || a.KB == 16) && a.t[0].subscales == nullptr) {
        int64_t want = (nt_total + 3 * cus - 1) / (3 * cus);
        if (want > kGemvMaxRT) want = kGemvMaxRT;
        grid64 = (nt_total + want - 1) / want;
    } else {
        int64_t want = (nt_total + cus - 1) / cus;
        if (want > kGemvMaxRT) want = kGemvMaxRT;
        grid64 = (nt_total + want - 1) / want;
        if (grid64 < cus && nt_total >= cus) grid64 = cus;  // (workgroups then own `want` or `want - 1` tiles)
    }
    if (grid64 > 0x7fffffff) return -2;
    const int grid = (int)grid64;
    const int rt = (int)((nt_total + grid - 1) / grid);
    a.nt_q = (int)(nt_total / grid);
    a.nt_r = (int)(nt_total % grid);
    switch (M) {
        case 1: return launch_blocks<1>(a, grid, rt, stream);
        case 2: return launch_blocks<2>(a, grid, rt, stream);
        default: return launch_blocks<4>(a, grid, rt, stream);
    }
}

template <int MP>
static int launch_rotated(const GemvArgs& a, int grid, int rt, hipStream_t stream) {
    const bool grouped = a.t[1].v_begin != 0x7fffffff;
    if (a.t[0].subscales != nullptr) {  // the sub-block variant: one tensor per launch
        switch (rt) {
            case 1: return launch_kernel<MP, 1, false, 0, true, true>(a, grid, stream);
            case 2: return launch_kernel<MP, 2, false, 0, true, true>(a, grid, stream);
            case 3: case 4: return launch_kernel<MP, 2, false, 0, true, true, 2>(a, grid, stream);
        }
        return -2;
    }
    switch (rt) {
        case 1: return grouped ? launch_kernel<MP, 1, true, 0, false, true>(a, grid, stream) : launch_kernel<MP, 1, false, 0, false, true>(a, grid, stream);
        case 2: return grouped ? launch_kernel<MP, 2, true, 0, false, true>(a, grid, stream) : launch_kernel<MP, 2, false, 0, false, true>(a, grid, stream);
        case 3: case 4: return grouped ? launch_kernel<MP, 2, true, 0, false, true, 2>(a, grid, stream) : launch_kernel<MP, 2, false, 0, false, true, 2>(a, grid, stream);
    }
    return -2;
}

int launch_gemv_rows(const GemvWeight* w, int count, int64_t K, const _Float16* Xt, const float* S, int64_t M, int MP, int y_f16,
                     uint32_t* flags, hipStream_t stream) {
    if (count < 1 || count > kGemvMaxGroup || M <= kGemvFusedMaxM || M > kGemvMaxM || (MP != 8 && MP != 16) || M > MP) return -2;
    GemvArgs a;
    a.X = Xt; a.S = S; a.flags = flags; a.ldx = 0; a.KB = (int)(K / kBlock); a.M = (int)M; a.y_f16 = y_f16;
    const int64_t nt_total = fill_tensors(a, w, count);
    if (nt_total < 0) return -2;
    // Every workgroup pulls all of the rotated activations (2 MP K bytes) through its compute unit's
    // L1: as many row tiles per workgroup as keep every compute unit busy, at most four (two steps of
    // two tiles per block).
    const int cus = cu_count();
    int64_t want = (nt_total + cus - 1) / cus;
    if (want > 4) want = 4;
    int64_t grid64 = (nt_total + want - 1) / want;
    if (grid64 < cus && nt_total >= cus) grid64 = cus;
    if (grid64 > 0x7fffffff) return -2;
    const int grid = (int)grid64;
    const int rt = (int)((nt_total + grid - 1) / grid);
    a.nt_q = (int)(nt_total / grid);
    a.nt_r = (int)(nt_total % grid);
    return MP == 8 ? launch_rotated<8>(a, grid, rt, stream) : launch_rotated<16>(a, grid, rt, stream);
}

}  // namespace itq3s
