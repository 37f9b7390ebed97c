// Tiled matmul for M > 16 activation rows (the prefill path): a dense contraction on the matrix
// cores.  Alg. 2 dequantizes a weight tile into on-chip memory and multiplies from there; here the
// tile written to LDS holds the un-rotated grid values d (q - z) in fp16 (exact for z = 0), the
// rotation having been moved to the activations (Sec. 2.3: <H v, x> = <v, H x>), so the tile loader
// needs two packed-fp16 operations per pair of weights and no butterflies.
//
//   Y[m][n] = sum_k x~[m][k'] * g[n][k']  -  sum_b d z 16 x[m][256 b],   g = d (c - 1)  (exact in fp16)
//
// The zero-point multiplies the sum of the rotated chunk, and H 1 = 16 e_0 makes that sum exactly
// 16 times the chunk's first element: the term is formed from the activations themselves in fp32.
// Folding z into the fp16 operand instead would multiply the rounding errors of x~ by z.  The term
// is rare (a fraction of a percent of the blocks on real weights), so the kernels note while they run
// whether a zero-point came by and only then walk the scale words of their columns at the end.
//
// k' is the channel order the unpack produces (within each group of 16 channels: 0,8,1,9,...,7,15);
// the rotation kernel writes x~ in the same order, so both LDS tiles are plain [row][k'].
//
// Workgroup: 256 threads = 2 x 2 wavefronts, tile 128 (m) x 128 (n) x 64 (k), wavefront tile 64 x 64
// as 2 x 2 v_mfma_f32_32x32x16_f16.  A operand = x~ rows, B operand = weight rows, so a lane's
// accumulator column is an output channel n and stores are contiguous along n.
#include <hip/hip_ext.h>

#include <type_traits>

#include "itq3s_dev.h"
#include "itq3s_kernels.h"

namespace itq3s {

constexpr int BM = 128, BN = 128, BK = 64;
// the 256 x 256 variant below takes over when there are enough rows to fill its tiles and enough
// tiles to occupy the chip
constexpr int kGemmBigMinM = 192, kGemmBigMinTiles = 128;
constexpr int LDT = BK + 8;  // LDS row stride in halves (padding keeps 16-byte reads conflict-free)

struct GemmArgs {
    const uint32_t* codes;
    const uint32_t* scales;
    const _Float16* Xt;  // [M][K] in k' order
    const _Float16* X;   // [M][ldx] the activations themselves (zero-point term)
    void* Y;
    uint32_t* flags;
    int64_t N, K, M, ldy, ldx;
    int NT, KB, y_f16;
};

// Zero-point term of one 32 x 32 output block that has already been stored: column n (this lane's),
// rows row0 + 8*(v/4) + 4*kg + v%4.  Walks the column's scale words and, for blocks with z != 0,
// subtracts d z 16 x[m][256 b] from the stored outputs (each output belongs to one lane).  Working
// on memory keeps the rare path out of the register budget of the main loop.
__device__ __forceinline__ void subtract_zero_points(const GemmArgs& a, int64_t n, int64_t row0, int kg) {
    if (n >= a.N) return;
    const uint32_t* sc = a.scales + (n >> 4) * a.KB * kTileRows + (n & 15);
#pragma unroll 1
    for (int b = 0; b < a.KB; ++b) {
        const uint32_t w = sc[(int64_t)b * kTileRows];
        const float z = f16_bits_to_f32(w >> 16);
        if (z != 0.f) {
            const float dz = f16_bits_to_f32(w & 0xffffu) * z;
#pragma unroll 1
            for (int v = 0; v < 16; ++v) {
                const int64_t m = row0 + 8 * (v >> 2) + 4 * kg + (v & 3);
                if (m < a.M) {
                    const float t = dz * (16.0f * (float)a.X[m * a.ldx + (int64_t)b * kBlock]);
                    if (a.y_f16) {
                        _Float16* y = reinterpret_cast<_Float16*>(a.Y) + m * a.ldy + n;
                        *y = (_Float16)((float)*y - t);
                    } else {
                        float* y = reinterpret_cast<float*>(a.Y) + m * a.ldy + n;
                        *y = *y - t;
                    }
                }
            }
        }
    }
}

__global__ __launch_bounds__(256) void gemm_kernel(const GemmArgs a) {
    __shared__ __align__(16) _Float16 As[BM * LDT];
    __shared__ __align__(16) _Float16 Bs[BN * LDT];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;  // wavefront position in the 2 x 2 arrangement
    const int64_t m0 = (int64_t)blockIdx.y * BM;
    const int nt0 = blockIdx.x * (BN / 16);
    const int KT = (int)(a.K / BK);

    // weight loader role: 16-row tile tl, row r, half p of the 64-channel quarter
    const int wp = tid & 1, wr = (tid >> 1) & 15, wtl = tid >> 5;
    const bool w_ok = nt0 + wtl < a.NT;
    // activation loader role: four 16-byte pieces per thread
    uint4 xa[4];
    uint2 wlo;
    uint32_t whi = 0, wsc = 0, bad = 0, any_z = 0;

    auto load_global = [&](int kt) {
        const int b = kt >> 2, q = kt & 3;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = tid + 256 * i, row = idx >> 3, c16 = idx & 7;
            const int64_t m = m0 + row;
            xa[i] = m < a.M ? *reinterpret_cast<const uint4*>(a.Xt + m * a.K + (int64_t)kt * BK + c16 * 8) : make_uint4(0, 0, 0, 0);
        }
        if (w_ok) {
            const int64_t tile = (int64_t)(nt0 + wtl) * a.KB + b;
            const uint32_t* t = a.codes + tile * kTileWords;
            const int ln = 16 * q + wr;
            wlo = *reinterpret_cast<const uint2*>(t + 4 * ln + 2 * wp);
            whi = t[kTileLoWords + 2 * ln + wp];
            wsc = a.scales[tile * kTileRows + wr];
        } else {
            wlo = make_uint2(0x55555555u, 0x55555555u);
            whi = 0;
            wsc = 0;
        }
    };

    auto store_lds = [&]() {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = tid + 256 * i, row = idx >> 3, c16 = idx & 7;
            *reinterpret_cast<uint4*>(&As[row * LDT + c16 * 8]) = xa[i];
        }
        bad |= whi;
        any_z |= (wsc >> 16) & 0x7fffu;
        // g = d * (c - 1): c * 2^-14 sits in bits 11:10 of each half after shift-and-mask
        const _Float16 d = __builtin_bit_cast(_Float16, (uint16_t)(wsc & 0xffffu));
        const half2v dd = {d, d};
        const half2v k14 = {(_Float16)16384.0f, (_Float16)16384.0f};
        const half2v off = {(_Float16)(-1.0f), (_Float16)(-1.0f)};
        const uint32_t w2[2] = {wlo.x, wlo.y};
        _Float16* dst = &Bs[(wtl * 16 + wr) * LDT + 32 * wp];
#pragma unroll
        for (int w = 0; w < 2; ++w) {
            uint32_t o[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int sh = 10 - 2 * j;
                const uint32_t bits = (sh >= 0 ? (w2[w] << sh) : (w2[w] >> (-sh))) & 0x0C000C00u;
                half2v h = __builtin_bit_cast(half2v, bits);
                h = (h * k14 + off) * dd;
                o[j] = __builtin_bit_cast(uint32_t, h);
            }
            *reinterpret_cast<uint4*>(dst + 16 * w) = make_uint4(o[0], o[1], o[2], o[3]);
            *reinterpret_cast<uint4*>(dst + 16 * w + 8) = make_uint4(o[4], o[5], o[6], o[7]);
        }
    };

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int l32 = lane & 31, kg = lane >> 5;
    load_global(0);
    for (int kt = 0; kt < KT; ++kt) {
        __syncthreads();
        store_lds();
        __syncthreads();
        if (kt + 1 < KT) load_global(kt + 1);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            half8 af[2], bf[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) af[i] = *reinterpret_cast<const half8*>(&As[(wm * 64 + i * 32 + l32) * LDT + ks * 16 + kg * 8]);
#pragma unroll
            for (int j = 0; j < 2; ++j) bf[j] = *reinterpret_cast<const half8*>(&Bs[(wn * 64 + j * 32 + l32) * LDT + ks * 16 + kg * 8]);
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
            const int64_t n = (int64_t)nt0 * 16 + wn * 64 + j * 32 + l32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t m = m0 + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
                if (m < a.M && n < a.N) {
                    if (a.y_f16) reinterpret_cast<_Float16*>(a.Y)[m * a.ldy + n] = (_Float16)acc[i][j][v];
                    else reinterpret_cast<float*>(a.Y)[m * a.ldy + n] = acc[i][j][v];
                }
            }
        }
    // zero-point term, only if some block of the workgroup's 128 rows has one
    if (__syncthreads_or(any_z != 0u)) {
#pragma unroll 1
        for (int ij = 0; ij < 4; ++ij) {
            const int i = ij >> 1, j = ij & 1;
            subtract_zero_points(a, (int64_t)nt0 * 16 + wn * 64 + j * 32 + l32, m0 + wm * 64 + i * 32, kg);
        }
    }
    if (a.flags != nullptr && bad != 0u) atomicOr(a.flags, kFlagBadCode);
}

// ------------------------------------------------------------------------------------------------
// Large-M variant: workgroup tile 256 (m) x 256 (n), eight wavefronts as 2 (m) x 4 (n), wavefront
// tile 128 x 64 = 4 x 2 v_mfma_f32_32x32x16_f16 (128 accumulator registers per lane, two wavefronts
// per SIMD so that one unpacks while the other multiplies).
//
// Only the activations go through LDS (two stages of 256 rows x 64 channels, one barrier per stage).
// The weights never do: a lane of the 32x32x16 product supplies, for its column n, eight consecutive
// channels k' of the step -- and one low-plane word of the packed tile holds exactly the 16 channels
// of one step of one row, in k' order after the shift-and-mask unpack (pairs (slot j, slot j+8)).
// So every lane loads the words of its own two rows (16 bytes = four steps per load), turns its
// half of a word into four half2 values d (c - 1) in registers, and feeds the matrix core.  The
// two wavefronts that share a column range repeat that unpack; in exchange the LDS carries half the
// traffic and the weight path needs no barrier.
//
// Tile order: workgroups are dealt to the 8 chiplets round-robin by the hardware, so chiplet x takes
// the contiguous run [x * per, (x+1) * per) of the tile list.  The list walks panels of two tile rows
// (512 activation rows), inside a panel column by column: the 32 workgroups that run together on one
// chiplet then cover 2 x 16 tiles and share, in that chiplet's L2, two activation slabs (the expensive
// operand: 2 bytes per element) among sixteen workgroups each and sixteen weight slabs (0.39 bytes per
// element) between two.
constexpr int GM = 256, GN = 256, GK = 64;
constexpr int GLD = GK + 8;  // LDS row stride in halves: 144 bytes, conflict-free for 16-byte reads
constexpr int GT = 512;      // threads
constexpr int kGemmBigLds = 2 * GM * GLD * 2;  // bytes, dynamic (above the 64 KB static limit)

__global__ __launch_bounds__(GT) void gemm_big_kernel(const GemmArgs a, int tiles_m, int tiles_n, int per_chiplet) {
    extern __shared__ __align__(16) _Float16 As[];  // [2][GM * GLD]

    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int t = xcd * per_chiplet + slot;
    if (slot >= per_chiplet || t >= tiles_m * tiles_n) return;
    constexpr int kPanel = 2;
    const int panel = t / (kPanel * tiles_n), within = t - panel * (kPanel * tiles_n);
    const int rows = tiles_m - panel * kPanel < kPanel ? tiles_m - panel * kPanel : kPanel;  // the last panel may be short
    const int tn = within / rows, tm = panel * kPanel + (within - tn * rows);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3;
    const int l32 = lane & 31, kg = lane >> 5;
    const int64_t m0 = (int64_t)tm * GM;
    const int64_t n0 = (int64_t)tn * GN;

    // Every load below is unconditional (rows past M or N and steps past K are clamped to valid
    // memory; what they produce lands in outputs that are never stored), so the loop is straight-line
    // and the load counter alone orders loads and use.
    // ---- activation loader: four 16-byte pieces per thread and stage (row = idx/8, piece = idx%8),
    // loaded one stage (four MFMA steps) before they are written to LDS
    u32x4 xa0, xa1, xa2, xa3;  // (plain variables: an array shared by two lambdas stays in memory)
    const int xr = tid >> 3, xc = tid & 7;  // rows xr, xr+64, xr+128, xr+192
    const _Float16* xrow[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) xrow[i] = a.Xt + (m0 + xr + 64 * i < a.M ? m0 + xr + 64 * i : a.M - 1) * a.K + xc * 8;
    const int KT = (int)(a.K / GK);
    auto load_x = [&](int kt) {
        const int k = (kt < KT ? kt : KT - 1) * GK;
        xa0 = *reinterpret_cast<const u32x4*>(xrow[0] + k);
        xa1 = *reinterpret_cast<const u32x4*>(xrow[1] + k);
        xa2 = *reinterpret_cast<const u32x4*>(xrow[2] + k);
        xa3 = *reinterpret_cast<const u32x4*>(xrow[3] + k);
    };
    auto store_x = [&](int stage) {
        _Float16* dst = As + stage * (GM * GLD) + xr * GLD + xc * 8;
        *reinterpret_cast<u32x4*>(dst) = xa0;
        *reinterpret_cast<u32x4*>(dst + 64 * GLD) = xa1;
        *reinterpret_cast<u32x4*>(dst + 128 * GLD) = xa2;
        *reinterpret_cast<u32x4*>(dst + 192 * GLD) = xa3;
    };

    // ---- weight loader: this lane's two rows n = n0 + wn*64 + j*32 + l32.  Row j sits 2j tile rows
    // below row 0; offsets are 32-bit, relative to the workgroup's first tile row (its 16 tile rows
    // span 16*KB tiles, far below 2^31 words for any K this library accepts).
    const int64_t nt0 = n0 >> 4;
    const uint32_t* const wg_codes = a.codes + nt0 * a.KB * kTileWords;
    const uint32_t* const wg_scales = a.scales + nt0 * a.KB * kTileRows;
    const int r16 = l32 & 15;
    uint32_t woff[2], soff[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        int64_t tr = wn * 4 + (l32 >> 4) + 2 * j;
        if (nt0 + tr > a.NT - 1) tr = a.NT - 1 - nt0;
        woff[j] = (uint32_t)tr * (uint32_t)a.KB * kTileWords + 4 * r16;
        soff[j] = (uint32_t)tr * (uint32_t)a.KB * kTileRows + r16;
    }
    uint32_t bad = 0;
    const int QT = KT;  // quarters of a block: 64 channels = one LDS stage = four MFMA steps
    uint2 hi0, hi1;  // high-plane words of the quarter in flight; folded into `bad` a stage later
    auto load_w = [&](int qt_, uint4 (&w)[2], uint32_t (&sc)[2]) {  // quarter of the row: block qt/4, quarter qt%4
        const int qt = qt_ < QT ? qt_ : QT - 1;
        const uint32_t b = (uint32_t)qt >> 2, q = (uint32_t)qt & 3;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint32_t* tile = wg_codes + (woff[j] + b * kTileWords);  // low-plane words of lane 16q + r16 start at + 64q
            w[j] = *reinterpret_cast<const uint4*>(tile + 64 * q);
            (j == 0 ? hi0 : hi1) = *reinterpret_cast<const uint2*>(tile + kTileLoWords + 32 * q - 2 * r16);
            sc[j] = wg_scales[soff[j] + b * kTileRows];
        }
    };
    // Unpack without shifts: the two code bits of pair p sit at bits 2p+1:2p of each half of the
    // word.  OR-ed into the mantissa of the half 2^(10-2p) (bit 2p of whose mantissa weighs exactly 1)
    // they form 2^(10-2p) + c; adding -(2^(10-2p) + 1) gives the digit c - 1 exactly, times d (exact).
    // One and-or, one add, one multiply per pair of weights.
    half2v dd[2];  // per row: d of the block being unpacked
    uint32_t any_z = 0;  // did one of this lane's rows see a zero-point?
    auto set_scale = [&](const uint32_t (&sc)[2]) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const _Float16 d = __builtin_bit_cast(_Float16, (uint16_t)(sc[j] & 0xffffu));
            dd[j] = half2v{d, d};
            any_z |= (sc[j] >> 16) & 0x7fffu;
        }
    };
    // word = the 16 channels of one MFMA step of row j; this lane's eight are the pairs 4kg .. 4kg+3
    auto unpack = [&](uint32_t word, int j) -> half8 {
        const uint32_t v = word >> (8 * kg);
        uint32_t o[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            constexpr uint32_t kMagic[4] = {0x64006400u, 0x5C005C00u, 0x54005400u, 0x4C004C00u};  // 1024, 256, 64, 16
            constexpr float kBase[4] = {1024.0f, 256.0f, 64.0f, 16.0f};
            uint32_t bits;
            asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(bits) : "v"(v), "s"(0x00030003u << (2 * p)), "v"(kMagic[p]));
            const _Float16 o1 = (_Float16)(-(kBase[p] + 1.0f));
            half2v h = __builtin_bit_cast(half2v, bits);
            h = (h + half2v{o1, o1}) * dd[j];
            o[p] = __builtin_bit_cast(uint32_t, h);
        }
        const uint4 u = make_uint4(o[0], o[1], o[2], o[3]);
        return __builtin_bit_cast(half8, u);
    };

    floatx16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // One MFMA step: 4 x 2 products on the fragments af (activations, read from LDS a step earlier)
    // and bf (weights), while the activation fragments of the next step are read into an and the
    // weights of the NEXT step (words nw0, nw1 of rows 0, 1) are unpacked into bf for the step after
    // -- the unpack belongs to no LDS stage, so that pipeline runs straight through the barriers.
    // The scheduling groups ask for the order: the LDS reads, then one matrix instruction and four
    // vector instructions, eight times.
    half8 bf[2];
    const _Float16* const a_lane = As + (wm * 128 + l32) * GLD + kg * 8;  // + stage*GM*GLD + i*32*GLD + ks*16
    auto read_a = [&](int stage, int ks, half8 (&af)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) af[i] = *reinterpret_cast<const half8*>(a_lane + stage * (GM * GLD) + i * 32 * GLD + ks * 16);
    };
    auto step = [&](const half8 (&af)[4], uint32_t nw0, uint32_t nw1) {
        const half8 n0v = unpack(nw0, 0), n1v = unpack(nw1, 1);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
        bf[0] = n0v;
        bf[1] = n1v;
    };
    auto interleave = [&](int ds_reads) {
        if (ds_reads) __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
        }
    };

    // Stage qt (64 channels = a quarter of a block) lives in LDS buffer qt & 1.  While it is
    // multiplied, the activations and the weights of stage qt+1 are on their way; the scheduling
    // fences keep the loads where they are written (the compiler would sink them next to their use
    // and wait for them at once).
    uint4 wcur[2], wnext[2];
    uint32_t sc_next[2];
    half8 af0[4], af1[4];
    load_x(0);
    load_w(0, wcur, sc_next);
    set_scale(sc_next);
    bad |= hi0.x | hi0.y | hi1.x | hi1.y;
    bf[0] = unpack(wcur[0].x, 0);
    bf[1] = unpack(wcur[1].x, 1);
    store_x(0);
    __syncthreads();
    for (int qt = 0; qt < QT; ++qt) {
        const int stage = qt & 1;
        load_x(qt + 1);
        load_w(qt + 1, wnext, sc_next);
        read_a(stage, 0, af0);
        __builtin_amdgcn_sched_barrier(0);
        read_a(stage, 1, af1);
        step(af0, wcur[0].y, wcur[1].y);
        interleave(1);
        __builtin_amdgcn_sched_barrier(0);
        read_a(stage, 2, af0);
        step(af1, wcur[0].z, wcur[1].z);
        interleave(1);
        __builtin_amdgcn_sched_barrier(0);
        read_a(stage, 3, af1);
        step(af0, wcur[0].w, wcur[1].w);
        interleave(1);
        __builtin_amdgcn_sched_barrier(0);
        set_scale(sc_next);  // the next quarter may start a new block
        bad |= hi0.x | hi0.y | hi1.x | hi1.y;
        __builtin_amdgcn_sched_barrier(0);
        step(af1, wnext[0].x, wnext[1].x);
        interleave(0);
        __builtin_amdgcn_sched_barrier(0);
        store_x(stage ^ 1);
#pragma unroll
        for (int j = 0; j < 2; ++j) wcur[j] = wnext[j];
        __syncthreads();
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
    // zero-point term, only if a lane of this wavefront met one (columns past N read clamped rows and
    // may trigger it needlessly; nothing is stored for them)
    if (__builtin_amdgcn_ballot_w64(any_z != 0u) != 0ull) {
#pragma unroll 1
        for (int ij = 0; ij < 8; ++ij) {
            const int i = ij >> 1, j = ij & 1;
            subtract_zero_points(a, n0 + wn * 64 + j * 32 + l32, m0 + wm * 128 + i * 32, kg);
        }
    }
    if (a.flags != nullptr && bad != 0u) atomicOr(a.flags, kFlagBadCode);
}

int launch_gemm(const uint32_t* codes, const uint32_t* scales, int64_t N, int64_t K, const _Float16* Xt, const _Float16* X, int64_t ldx,
                int64_t M, void* Y, int y_f16, int64_t ldy, uint32_t* flags, hipStream_t stream) {
    GemmArgs a;
    a.codes = codes; a.scales = scales; a.Xt = Xt; a.X = X; a.ldx = ldx; a.Y = Y; a.flags = flags;
    a.N = N; a.K = K; a.M = M; a.ldy = ldy; a.NT = (int)((N + 15) / 16); a.KB = (int)(K / kBlock); a.y_f16 = y_f16;
    const LaunchTiming tm = take_launch_timing();
    const int64_t tiles_m = (M + GM - 1) / GM, tiles_n = (N + GN - 1) / GN;
    if (M >= kGemmBigMinM && tiles_m * tiles_n >= kGemmBigMinTiles && tiles_m * tiles_n < 0x7fffffff / 8) {
        const int per = (int)((tiles_m * tiles_n + 7) / 8);
        const dim3 g((unsigned)(per * 8));
        static bool lds_limit_raised = false;
        if (!lds_limit_raised) {
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_big_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kGemmBigLds) != hipSuccess) return -6;
            lds_limit_raised = true;
        }
        if (tm.start != nullptr) hipExtLaunchKernelGGL(gemm_big_kernel, g, dim3(GT), kGemmBigLds, stream, tm.start, tm.stop, 0, a, (int)tiles_m, (int)tiles_n, per);
        else hipLaunchKernelGGL(gemm_big_kernel, g, dim3(GT), kGemmBigLds, stream, a, (int)tiles_m, (int)tiles_n, per);
        return hipGetLastError() == hipSuccess ? 0 : -6;
    }
    dim3 grid((unsigned)((N + BN - 1) / BN), (unsigned)((M + BM - 1) / BM));
    if (tm.start != nullptr) hipExtLaunchKernelGGL(gemm_kernel, grid, dim3(256), 0, stream, tm.start, tm.stop, 0, a);
    else hipLaunchKernelGGL(gemm_kernel, grid, dim3(256), 0, stream, a);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

}  // namespace itq3s
