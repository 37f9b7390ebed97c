// Tiled matmul for M > 16 activation rows (the prefill path): a dense contraction on the matrix
// cores.  Alg. 2 dequantizes a weight tile into on-chip memory and multiplies from there; here the
// operand fed to the matrix cores holds the un-rotated grid values d (q - z) in fp16 (exact for
// z = 0), the rotation having been moved to the activations (Sec. 2.3: <H v, x> = <v, H x>), so the
// weight path needs three packed-fp16 operations per pair of weights and no butterflies.
//
//   Y[m][n] = sum_k x~[m][k'] * g[n][k']  -  sum_b d z 16 x[m][256 b],   g = d (c - 1)  (exact in fp16)
//
// The zero-point multiplies the sum of the rotated chunk, and H 1 = 16 e_0 makes that sum exactly
// 16 times the chunk's first element: the term is formed from the activations themselves in fp32.
// Folding z into the fp16 operand instead would multiply the rounding errors of x~ by z.  The term
// is rare (a fraction of a percent of the blocks on real weights), so the kernel notes while it runs
// whether a zero-point came by and only then walks the scale words of its columns at the end; the
// terms are subtracted from the accumulators, so an output element is rounded once.
//
// k' is the channel order the unpack produces (within each group of 16 channels: 0,8,1,9,...,7,15);
// the rotation kernel writes x~ in the same order.  A operand = x~ rows, B operand = weight rows, so
// a lane's accumulator column is an output channel n and stores are contiguous along n.
#include <hip/hip_ext.h>

#include <type_traits>

#include "itq3s_dev.h"
#include <atomic>

#include "itq3s_kernels.h"

namespace itq3s {

constexpr int64_t kGemmMaxK = 1 << 22;  // per-lane byte offsets (up to 128 rows x K x 2) are 32-bit

struct GemmArgs {
    const uint32_t* codes;
    const uint32_t* scales;
    const _Float16* Xt;  // [M][K] in k' order
    const _Float16* X;   // [M][ldx] the activations themselves (zero-point term)
    void* Y;
    uint32_t* flags;
    int64_t N, K, M, ldy, ldx;
    int NT, KB, y_f16;
    // split-K (splits > 1): the contraction kernel writes partial tiles [tile][split][32][256 threads]
    // of four floats and ORs 1 into zflags[tile] if it met a zero-point; a second launch adds them up
    float* partial;
    uint32_t* zflags;
    int splits;
};

// LDS accesses by raw byte address, hidden from the compiler like every other LDS read of this file
// (it would order visible LDS accesses after all outstanding global -> LDS copies).
__device__ __forceinline__ void lds_write_b32(uint32_t addr, uint32_t v) { asm volatile("ds_write_b32 %0, %1" ::"v"(addr), "v"(v) : "memory"); }
__device__ __forceinline__ void lds_add_f32(uint32_t addr, float v) { asm volatile("ds_add_f32 %0, %1" ::"v"(addr), "v"(v) : "memory"); }
__device__ __forceinline__ uint32_t lds_read_f32_bits_now(uint32_t addr) {
    uint32_t r;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(r) : "v"(addr) : "memory");
    return r;
}
__device__ __forceinline__ float lds_read_f32_now(uint32_t addr) {
    float r;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(r) : "v"(addr) : "memory");
    return r;
}

// Zero-point terms of a wavefront's output block, columns n_first .. n_first + 63, rows m_first ..
// m_first + ROWS - 1, summed in fp32 into a wavefront-private LDS table (ROWS x 64 floats at byte
// address `table`; element (row, col) at word 64 row + (col + row) % 64, which spreads a column over
// the banks) -- they are subtracted from the accumulators BEFORE the output is rounded: with fp16
// outputs, correcting the stored value instead would round a sum that still contains the +z offset of
// every code and lose up to 2^-11 of that larger number.  Lane l walks the scale words of column
// n_first + l, sixteen blocks per batch (independent loads).  For each block with z != 0 -- a fraction
// of a percent on real weights -- the whole wavefront adds d z 16 x[m][256 b] to that column of the
// table, one row per lane.  Per element the blocks are added in ascending order by one lane at a
// time, so the result does not depend on scheduling.
template <int ROWS>
__device__ __forceinline__ void zero_point_terms(const GemmArgs& a, int64_t n_first, int64_t m_first, int lane, uint32_t table) {
#pragma unroll 8
    for (int i = 0; i < ROWS; ++i) lds_write_b32(table + (uint32_t)(i * 64 + lane) * 4u, 0u);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    const int64_t n = n_first + lane;
    const int64_t nc = n < a.N ? n : a.N - 1;
    const uint32_t* sc = a.scales + (nc >> 4) * a.KB * kTileRows + (nc & 15);
#pragma unroll 1
    for (int b0 = 0; b0 < a.KB; b0 += 16) {
        uint32_t w[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) w[u] = sc[(int64_t)(b0 + u < a.KB ? b0 + u : a.KB - 1) * kTileRows];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const bool hit = (w[u] & 0x7fff0000u) != 0u && n < a.N && b0 + u < a.KB;
            unsigned long long todo = __builtin_amdgcn_ballot_w64(hit);
            while (todo != 0ull) {  // uniform
                const int src = __builtin_ctzll(todo);
                todo &= todo - 1ull;
                const uint32_t word = (uint32_t)__builtin_amdgcn_readlane((int)w[u], src);
                const float dz = f16_bits_to_f32(word & 0xffffu) * f16_bits_to_f32(word >> 16);
#pragma unroll 1
                for (int r = 0; r < ROWS; r += kWave) {
                    const int row = r + lane;
                    const int64_t m = m_first + row;
                    if (m < a.M && row < ROWS) {
                        const float t = dz * (16.0f * (float)a.X[m * a.ldx + (int64_t)(b0 + u) * kBlock]);
                        lds_add_f32(table + (uint32_t)(row * 64 + ((src + row) & 63)) * 4u, t);
                    }
                }
            }
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
}

// The common case of the above -- the zero-points of a wavefront's 64 columns sit in at most eight of
// them -- needs no table of all columns: one 128-row strip of floats per such column (strip_offset())
// fits the wavefront's own corner of the weight ring (1 KiB of each of its four stages: two strips
// each), so nothing is shared, nobody is waited for, and one scan serves all 128 rows.  cols receives
// the columns (0..63, -1: slot unused).  Returns false, with the strips in an undefined state, if a
// ninth column turns up.
constexpr int kStrips = 8;
struct StripColumns {
    int c[kStrips];
};
__device__ __forceinline__ uint32_t strip_offset(int slot) { return (uint32_t)((slot >> 1) * 4096 + (slot & 1) * 512); }
__device__ __forceinline__ bool zero_point_terms_few_columns(const GemmArgs& a, int64_t n_first, int64_t m_first, int lane, uint32_t strips,
                                                             StripColumns& cols) {
#pragma unroll
    for (int s = 0; s < kStrips; ++s) {
        cols.c[s] = -1;
        lds_write_b32(strips + strip_offset(s) + (uint32_t)(4 * lane), 0u);
        lds_write_b32(strips + strip_offset(s) + (uint32_t)(4 * (lane + 64)), 0u);
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    const int64_t n = n_first + lane;
    const int64_t nc = n < a.N ? n : a.N - 1;
    const uint32_t* sc = a.scales + (nc >> 4) * a.KB * kTileRows + (nc & 15);
#pragma unroll 1
    for (int b0 = 0; b0 < a.KB; b0 += 16) {
        uint32_t w[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) w[u] = sc[(int64_t)(b0 + u < a.KB ? b0 + u : a.KB - 1) * kTileRows];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const bool hit = (w[u] & 0x7fff0000u) != 0u && n < a.N && b0 + u < a.KB;
            unsigned long long todo = __builtin_amdgcn_ballot_w64(hit);
            while (todo != 0ull) {  // uniform
                const int src = __builtin_ctzll(todo);
                todo &= todo - 1ull;
                // the column's slot, or the first free one (uniform; static indices only)
                int slot = -1;
#pragma unroll
                for (int q = kStrips - 1; q >= 0; --q) slot = cols.c[q] == src ? q : slot;
                if (slot < 0) {
#pragma unroll
                    for (int q = kStrips - 1; q >= 0; --q) slot = cols.c[q] < 0 ? q : slot;
                    if (slot < 0) return false;
#pragma unroll
                    for (int q = 0; q < kStrips; ++q) cols.c[q] = q == slot ? src : cols.c[q];
                }
                const uint32_t word = (uint32_t)__builtin_amdgcn_readlane((int)w[u], src);
                const float dz = f16_bits_to_f32(word & 0xffffu) * f16_bits_to_f32(word >> 16);
#pragma unroll
                for (int r = 0; r < 128; r += kWave) {
                    const int row = r + lane;
                    const int64_t m = m_first + row;
                    if (m < a.M) {
                        const float t = dz * (16.0f * (float)a.X[m * a.ldx + (int64_t)(b0 + u) * kBlock]);
                        lds_add_f32(strips + strip_offset(slot) + (uint32_t)(4 * row), t);
                    }
                }
            }
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    return true;
}

// ------------------------------------------------------------------------------------------------
// Workgroup tile 128 (m) x 256 (n), four wavefronts side by side along n, wavefront tile 128 x 64 =
// 4 x 2 v_mfma_f32_32x32x16_f16 (128 accumulator registers per lane), K in quarters of a block
// (64 channels = four MFMA steps), one barrier per quarter.  Two workgroups share a compute unit
// (68 KiB of LDS, about 220 registers), so every SIMD holds two wavefronts from different workgroups:
// one unpacks while the other multiplies, and their barriers are not aligned.
// (A 256 x 256 tile with eight wavefronts, one workgroup per compute unit, was measured too: within
// 3 % where tiles are plentiful, up to 40 % slower where they are not.)
//
// A lane of the 32x32x16 product supplies, for its column n, eight consecutive channels k' of the
// step -- and one low-plane word of the packed tile holds exactly the 16 channels of one step of one
// row, in k' order after the unpack (pairs (slot j, slot j+8)).  So a lane needs, per quarter, the
// four words (16 bytes) of each of its two rows, turns its half of a word into four half2 values
// d (c - 1) in registers, and feeds the matrix core; no dequantized tile is ever stored.
//
// Every operand is copied global -> LDS by the memory pipe itself (buffer_load ... lds: no registers,
// no LDS store instructions), two to three quarters ahead of the arithmetic -- about 1.5 us of lead,
// which covers an HBM miss.
//
// LDS (68 KiB):
//   activations  ring of 3 quarters x 128 rows x 128 bytes, no padding (one copy instruction writes
//                1 KiB = 8 rows, lane l the 16-byte piece l of it).  To keep the 16-byte fragment
//                reads conflict-free, piece p of row r holds channel chunk p ^ swz(r),
//                swz(r) = (r & 7) ^ ((r >> 3) & 1): sixteen consecutive rows reading the same chunk
//                touch sixteen different 16-byte groups of 256 bytes, eight rows eight groups of 128.
//   weights      ring of 4 quarters x 4 wavefronts x 1 KiB: lane (l32, kg) copies the 16 bytes of ITS
//                row j = kg, and later reads both rows (its own piece and that of lane (l32, 1 - kg)).
//                Private to the wavefront: ordered by the load counter alone, no barrier.
//   scales       ring of 4 quarters x 4 wavefronts x 256 bytes, same pattern with 4 bytes per lane.
// The weight ring runs one quarter further ahead than the activation ring because the last MFMA step
// of a quarter already unpacks the first words of the next one.
//
// All LDS reads are written as inline instructions with their own counter waits: the compiler orders
// every LDS read it can see after ALL outstanding global -> LDS copies, which would drain the
// look-ahead at the first read of each quarter.  Since no load returns into registers, it inserts no
// load-counter waits of its own inside the loop either; the explicit ones are all there are.
//
// Tile order: workgroups are dealt to the 8 chiplets round-robin by the hardware, so chiplet x takes
// the contiguous run [x * per, (x+1) * per) of the tile list.  The list walks panels of four tile
// rows (512 activation rows), inside a panel column by column: the workgroups that run together on
// one chiplet then cover 4 x 16 tiles and share, in that chiplet's L2, four activation slabs (the
// expensive operand: 2 bytes per element) among sixteen workgroups each and sixteen weight slabs
// (0.39 bytes per element) among four.
constexpr int GM = 128, GN = 256, GK = 64;
constexpr int GT = 256;  // threads
constexpr int kXStages = 3, kWStages = 4;
constexpr int kXStageBytes = GM * GK * 2;                   // 16384
constexpr int kWRingBase = kXStages * kXStageBytes;         // 49152
constexpr int kWStageBytes = 4 * 1024;                      // 4 wavefronts x 64 lanes x 16 bytes
constexpr int kSRingBase = kWRingBase + kWStages * kWStageBytes;  // 65536
constexpr int kSStageBytes = 4 * 256;                       // 4 wavefronts x 64 lanes x 4 bytes
constexpr int kDoneWord = kSRingBase + kWStages * kSStageBytes;   // 69632: count of wavefronts that are done with the rings
constexpr int kGemmLds = kDoneWord + 16;
constexpr int kPanel = 4;                                   // tile rows per panel

template <int OFF>
__device__ __forceinline__ half8 lds_read_b128(uint32_t addr) {
    half8 r;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF) : "memory");
    return r;
}
template <int OFF>
__device__ __forceinline__ u32x4 lds_read_u4(uint32_t addr) {
    u32x4 r;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF) : "memory");
    return r;
}
template <int OFF>
__device__ __forceinline__ uint32_t lds_read_b32(uint32_t addr) {
    uint32_t r;
    asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF) : "memory");
    return r;
}
// wait until at most N LDS reads are outstanding; the values are passed through so that no use of
// them can be scheduled ahead of the wait
#define ITQ3S_LDS_WAIT(N, af) asm volatile("s_waitcnt lgkmcnt(" #N ")" : "+v"(af[0]), "+v"(af[1]), "+v"(af[2]), "+v"(af[3]))

// Position of tile t in the walk described above.
__device__ __forceinline__ void tile_coords(int t, int tiles_m, int tiles_n, int& tm, int& tn) {
    const int panel = t / (kPanel * tiles_n), within = t - panel * (kPanel * tiles_n);
    const int rows = tiles_m - panel * kPanel < kPanel ? tiles_m - panel * kPanel : kPanel;  // the last panel may be short
    tn = within / rows;
    tm = panel * kPanel + (within - tn * rows);
}

// Store 32 rows (m_first ..) of a wavefront's 64 columns (n0 + 64 wn ..).  Accumulator register v of a
// 32x32 block: row = 8*(v/4) + 4*(lane/32) + v%4, column = lane%32.  kTerms: minus the zero-point
// terms of these rows, which start at row `row0` of the wavefront's LDS table (zero_point_terms()).
template <int kTerms>  // 0: none; 1: table of all columns (row0: its row of m_first); 2: strips of a few columns (row0 likewise)
__device__ __forceinline__ void store_rows(const GemmArgs& a, const floatx16 (&acc)[2], int64_t m_first, int64_t n0, int wn, int lane,
                                           int row0 = 0, uint32_t table = 0, const StripColumns* cols = nullptr) {
    const int l32 = lane & 31, kg = lane >> 5;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int64_t n = n0 + wn * 64 + j * 32 + l32;
        floatx16 terms;
        if constexpr (kTerms != 0) {
            const int col = 32 * j + l32;
            int slot = -1;  // (strips only)
            if constexpr (kTerms == 2) {
#pragma unroll
                for (int q = 0; q < kStrips; ++q) slot = cols->c[q] == col ? q : slot;
            }
            // sixteen reads in flight, one wait
            uint32_t t[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + 8 * (v >> 2) + 4 * kg + (v & 3);
                const uint32_t addr = kTerms == 1 ? table + (uint32_t)(row * 64 + ((col + row) & 63)) * 4u
                                                  : table + strip_offset(slot < 0 ? 0 : slot) + (uint32_t)(4 * row);
                asm volatile("ds_read_b32 %0, %1" : "=v"(t[v]) : "v"(addr) : "memory");
            }
            asm volatile("s_waitcnt lgkmcnt(0)"
                         : "+v"(t[0]), "+v"(t[1]), "+v"(t[2]), "+v"(t[3]), "+v"(t[4]), "+v"(t[5]), "+v"(t[6]), "+v"(t[7]), "+v"(t[8]), "+v"(t[9]),
                           "+v"(t[10]), "+v"(t[11]), "+v"(t[12]), "+v"(t[13]), "+v"(t[14]), "+v"(t[15]));
#pragma unroll
            for (int v = 0; v < 16; ++v) terms[v] = (kTerms == 2 && slot < 0) ? 0.0f : __builtin_bit_cast(float, t[v]);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int64_t m = m_first + 8 * (v >> 2) + 4 * kg + (v & 3);
            if (m < a.M && n < a.N) {
                float y = acc[j][v];
                if constexpr (kTerms != 0) y = y - terms[v];
                if (a.y_f16) reinterpret_cast<_Float16*>(a.Y)[m * a.ldy + n] = (_Float16)y;
                else reinterpret_cast<float*>(a.Y)[m * a.ldy + n] = y;
            }
        }
    }
}

// Store a wavefront's 128 x 64 block (rows m0.., columns n0 + 64 wn ..).
__device__ __forceinline__ void store_tile(const GemmArgs& a, const floatx16 (&acc)[4][2], int64_t m0, int64_t n0, int wn, int lane) {
#pragma unroll
    for (int i = 0; i < 4; ++i) store_rows<0>(a, acc[i], m0 + i * 32, n0, wn, lane);
}

// (two wavefronts per SIMD: at most 256 registers)
__global__ __launch_bounds__(GT) __attribute__((amdgpu_waves_per_eu(2, 2))) void gemm_kernel(const GemmArgs a, int tiles_m, int tiles_n, int per_chiplet) {
    extern __shared__ __align__(1024) char lds[];
    // LDS byte address of the buffer, for the read instructions below that take raw addresses
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;

    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int item = xcd * per_chiplet + slot;
    if (slot >= per_chiplet || item >= tiles_m * tiles_n * a.splits) return;
    // the splits of a tile are neighbours in the list
    const int t = item / a.splits, split = item - t * a.splits;
    int tm, tn;
    tile_coords(t, tiles_m, tiles_n, tm, tn);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave;
    const int l32 = lane & 31, kg = lane >> 5;
    const int64_t m0 = (int64_t)tm * GM;
    const int64_t n0 = (int64_t)tn * GN;
    const int KT = (int)(a.K / GK);
    // this workgroup's share of K: whole blocks, quarters q0 .. q1 - 1
    const int q0 = 4 * (int)((int64_t)split * a.KB / a.splits), q1 = 4 * (int)((int64_t)(split + 1) * a.KB / a.splits);

    // All copies go through buffer descriptors: a 32-bit per-lane offset fixed for the whole kernel
    // plus a scalar offset that advances with the stage -- no address arithmetic in the vector pipe.
    // Steps past the end of K repeat the last stage (valid memory, never consumed).
    constexpr int kRsrcFlags = 0x00027000;  // raw buffer, 32-bit elements
    // ---- activations: wavefront w copies pieces 4w .. 4w+3 of a stage (8 rows each); lane l supplies
    // row l/8 of the piece and the chunk that belongs at position l%8 of that row.  Rows past M read
    // row M-1 (their outputs are never stored).
    const __amdgpu_buffer_rsrc_t x_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<_Float16*>(a.Xt + m0 * a.K), 0, (int)(GM * a.K * 2), kRsrcFlags);
    int xoff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int64_t row = 8 * (4 * wave + i) + (lane >> 3);
        if (m0 + row > a.M - 1) row = a.M - 1 - m0;
        const int chunk = (lane & 7) ^ (lane >> 3) ^ (i & 1);
        xoff[i] = (int)(row * a.K * 2 + chunk * 16);
    }
    // ---- weights: the lane's OWN row n = n0 + wn*64 + kg*32 + l32, as byte offsets from the
    // workgroup's first tile row (16 tile rows x KB tiles: far below 2^31 bytes for any K accepted here)
    const int64_t nt0 = n0 >> 4;
    const int64_t wg_tile_rows = a.NT - nt0 < 16 ? a.NT - nt0 : 16;
    const __amdgpu_buffer_rsrc_t c_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint32_t*>(a.codes + nt0 * a.KB * kTileWords), 0, (int)(wg_tile_rows * a.KB * kTileWords * 4), kRsrcFlags);
    const __amdgpu_buffer_rsrc_t s_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint32_t*>(a.scales + nt0 * a.KB * kTileRows), 0, (int)(wg_tile_rows * a.KB * kTileRows * 4), kRsrcFlags);
    int woff, soff;
    {
        const int r16 = l32 & 15;
        int64_t tr = wn * 4 + (l32 >> 4) + 2 * kg;
        if (nt0 + tr > a.NT - 1) tr = a.NT - 1 - nt0;
        woff = (int)(tr * a.KB * kTileWords + 4 * r16) * 4;  // low-plane words of storage lane 16 q + r16: + 256 q bytes
        soff = (int)(tr * a.KB * kTileRows + r16) * 4;
    }
    auto copy_x = [&](int kt, int ring) {
        const int k_bytes = (kt < KT ? kt : KT - 1) * (GK * 2);
        char* dst = lds + ring * kXStageBytes + 4096 * wave;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(x_rsrc, (__attribute__((address_space(3))) void*)(dst + 1024 * i), 16, xoff[i], k_bytes, 0, 0);
    };
    auto copy_w = [&](int kt_) {  // quarter kt of the rows: block kt/4, quarter kt%4; ring position kt%4
        const int kt = kt_ < KT ? kt_ : KT - 1;
        const int b = kt >> 2, q = kt & 3, ring = kt_ & 3;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(c_rsrc, (__attribute__((address_space(3))) void*)(lds + kWRingBase + ring * kWStageBytes + 1024 * wave),
                                                 16, woff, b * (kTileWords * 4) + 256 * q, 0, 0);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(s_rsrc, (__attribute__((address_space(3))) void*)(lds + kSRingBase + ring * kSStageBytes + 256 * wave),
                                                 4, soff, b * (kTileRows * 4), 0, 0);
    };

    // ---- fragment reads: row i*32 + l32, chunk 2 ks + kg, at position chunk ^ swz(row);
    // swz depends on l32 only, so one byte offset per step ks serves all four i (+ 4096 i)
    uint32_t aoff[4];
    {
        const int s = (l32 & 7) ^ ((l32 >> 3) & 1);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) aoff[ks] = lds_base + (uint32_t)(l32 * 128 + (((2 * ks + kg) ^ s) * 16));
    }
    const uint32_t wread = lds_base + (uint32_t)(kWRingBase + 1024 * wave + 16 * l32);  // row 0 here, row 1 at + 512
    const uint32_t sread = lds_base + (uint32_t)(kSRingBase + 256 * wave + 4 * l32);    // row 0 here, row 1 at + 128

    uint32_t any_z = 0;
    half2v dd[2];
    auto set_scale = [&](uint32_t s0, uint32_t s1) {
        const _Float16 d0 = __builtin_bit_cast(_Float16, (uint16_t)(s0 & 0xffffu)), d1 = __builtin_bit_cast(_Float16, (uint16_t)(s1 & 0xffffu));
        dd[0] = half2v{d0, d0};
        dd[1] = half2v{d1, d1};
        any_z |= ((s0 | s1) >> 16) & 0x7fffu;
    };
    // Unpack without shifts: the two code bits of pair p sit at bits 2p+1:2p of each half of the
    // word.  OR-ed into the mantissa of the half 2^(10-2p) (bit 2p of whose mantissa weighs exactly 1)
    // they form 2^(10-2p) + c; adding -(2^(10-2p) + 1) gives the digit c - 1 exactly, times d (exact).
    // One and-or, one add, one multiply per pair of weights.
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

    half8 bf[2];
    auto step = [&](const half8 (&af)[4], uint32_t nw0, uint32_t nw1) {
        const half8 n0v = unpack(nw0, 0), n1v = unpack(nw1, 1);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
        bf[0] = n0v;
        bf[1] = n1v;
    };
    auto interleave = [&]() {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
        }
    };
    half8 af0[4], af1[4];
    auto read_a = [&](uint32_t addr, half8 (&af)[4]) {
        af[0] = lds_read_b128<0>(addr);
        af[1] = lds_read_b128<4096>(addr);
        af[2] = lds_read_b128<8192>(addr);
        af[3] = lds_read_b128<12288>(addr);
    };

    // The loop is rotated by one MFMA step: a trip starts right after a barrier with the LAST step of
    // the previous quarter (its fragments are already in registers), so that the matrix cores have
    // work while the first fragment reads of the new quarter are on their way, then runs steps 0..2
    // of its own quarter and ends with the barrier.  By then every wavefront has read the last
    // fragments of the quarter (they sit in registers), so its buffer is free for the copies issued
    // at the top of the next trip.
    //   trip q:  copies X(q+2), W(q+3) | read A(q,0) | [step (q-1,3)] | read A(q,1), W(q+1) |
    //            step (q,0) | read A(q,2) | step (q,1) | read A(q,3) | step (q,2) | waits, barrier
    // kFirst: there is no previous quarter (bf already holds the operands of step (q,0)).
    auto run_trip = [&](int q, int xr, auto first, const u32x4& c0, const u32x4& c1, u32x4& n0w, u32x4& n1w) {
        constexpr bool kFirst = decltype(first)::value;
        {
            const int xd = xr == 0 ? 2 : xr - 1;  // (q + 2) % 3: held quarter q-1, all of whose reads completed before the barrier
            copy_x(q + 2, xd);
            copy_w(q + 3);  // that slot held quarter q-1, read by this wavefront a trip ago
        }
        const uint32_t wr = wread + (uint32_t)(((q + 1) & 3) * kWStageBytes), sr = sread + (uint32_t)(((q + 1) & 3) * kSStageBytes);
        const uint32_t sb = (uint32_t)(xr * kXStageBytes);
        __builtin_amdgcn_sched_barrier(0);
        read_a(aoff[0] + sb, af0);
        if constexpr (!kFirst) {
            // last step of the previous quarter: fragments in af1 (read before the barrier); unpacks the
            // first words of this quarter, whose scale was set a trip ago
            step(af1, c0.x, c1.x);
            interleave();
            __builtin_amdgcn_sched_barrier(0);
        }
        n0w = lds_read_u4<0>(wr);
        n1w = lds_read_u4<512>(wr);
        uint32_t s0 = lds_read_b32<0>(sr), s1 = lds_read_b32<128>(sr);
        read_a(aoff[1] + sb, af1);
        asm volatile("s_waitcnt lgkmcnt(8)" : "+v"(af0[0]), "+v"(af0[1]), "+v"(af0[2]), "+v"(af0[3]));
        step(af0, c0.y, c1.y);
        interleave();
        __builtin_amdgcn_sched_barrier(0);
        read_a(aoff[2] + sb, af0);
        asm volatile("s_waitcnt lgkmcnt(4)"
                     : "+v"(af1[0]), "+v"(af1[1]), "+v"(af1[2]), "+v"(af1[3]), "+v"(n0w), "+v"(n1w), "+v"(s0), "+v"(s1));
        step(af1, c0.z, c1.z);
        interleave();
        __builtin_amdgcn_sched_barrier(0);
        read_a(aoff[3] + sb, af1);
        ITQ3S_LDS_WAIT(4, af0);
        step(af0, c0.w, c1.w);
        interleave();
        __builtin_amdgcn_sched_barrier(0);
        set_scale(s0, s1);  // for the unpack of the next quarter's first words, at the top of the next trip
        ITQ3S_LDS_WAIT(0, af1);
        // Everything issued before this trip's six copies has landed: the activations of quarter q+1
        // and the weights of quarter q+2 among them (copies complete in order).
        asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
        __builtin_amdgcn_s_barrier();
    };

    // Prologue: quarters 0 and 1 of everything and quarter 2 of the weights, in two groups of six
    // copies, so that waiting for all but six leaves exactly the second group in flight.
    u32x4 wa0, wa1, wb0, wb1;
    copy_x(q0, 0);
    copy_w(q0);
    __builtin_amdgcn_sched_barrier(0);
    copy_x(q0 + 1, 1);
    copy_w(q0 + 1);
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
    copy_w(q0 + 2);
    __builtin_amdgcn_sched_barrier(0);
    {
        wa0 = lds_read_u4<0>(wread);
        wa1 = lds_read_u4<512>(wread);
        uint32_t s0 = lds_read_b32<0>(sread), s1 = lds_read_b32<128>(sread);
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(wa0), "+v"(wa1), "+v"(s0), "+v"(s1));
        set_scale(s0, s1);
        bf[0] = unpack(wa0.x, 0);
        bf[1] = unpack(wa1.x, 1);
    }
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt vmcnt(2)" ::: "memory");  // quarter 1 has landed as well; only the two copies of copy_w(2) may be in flight
    if (tid == 0) {
        lds_write_b32(lds_base + kDoneWord, 0u);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
    __builtin_amdgcn_s_barrier();
    // The two register sets of the weights alternate by name, so trips come in pairs: the first trip
    // on its own, pairs (1,2), (3,4), ..., and the last trip (K is a multiple of 256: the number of
    // quarters is a multiple of four, so it is odd-numbered).
    run_trip(q0, 0, std::true_type{}, wa0, wa1, wb0, wb1);
    int xr = 1;
    for (int q = q0 + 1; q + 1 < q1; q += 2) {
        run_trip(q, xr, std::false_type{}, wb0, wb1, wa0, wa1);
        xr = xr == 2 ? 0 : xr + 1;
        run_trip(q + 1, xr, std::false_type{}, wa0, wa1, wb0, wb1);
        xr = xr == 2 ? 0 : xr + 1;
    }
    run_trip(q1 - 1, xr, std::false_type{}, wb0, wb1, wa0, wa1);
    // last step of the last quarter (the words it unpacks are never used)
    step(af1, wa0.x, wa1.x);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the look-ahead copies past the last quarter still target this workgroup's LDS
    // ... and this wavefront reads the rings no more.  Counted rather than met at a barrier: only a
    // wavefront that needs the rings' space for its zero-point table waits for the other three, and
    // every wavefront gets here without waiting for anything.
    if (lane == 0) asm volatile("ds_add_u32 %0, %1" ::"v"(lds_base + kDoneWord), "v"(1u) : "memory");

    // Format check, apart from the arithmetic: the high plane of the workgroup's 16 tile rows must be
    // zero (128 words per tile, a quarter of the packed bytes, read once more here).
    if (a.flags != nullptr && tm == 0 && split == 0) {  // once per tile column
        const uint4* hp = reinterpret_cast<const uint4*>(a.codes + nt0 * a.KB * kTileWords);
        const int64_t tiles = wg_tile_rows * a.KB;  // 32 pieces of 16 bytes per tile, at word 256 of each
        uint32_t bad = 0;
#pragma unroll 2
        for (int64_t i = tid; i < tiles * 32; i += GT) {
            const uint4 v = hp[(i >> 5) * (kTileWords / 4) + kTileLoWords / 4 + (i & 31)];
            bad |= v.x | v.y | v.z | v.w;
        }
        if (bad != 0u) atomicOr(a.flags, kFlagBadCode);
    }
    const bool zero_points = __builtin_amdgcn_ballot_w64(any_z != 0u) != 0ull;  // did a lane of this wavefront meet one?
    if (a.splits > 1) {
        // split-K: park the sums; the launch that follows adds the shares of every tile in split order
        floatx4* const mine = reinterpret_cast<floatx4*>(a.partial) + ((int64_t)(t * a.splits + split) * 32) * GT + tid;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    mine[((i * 2 + j) * 4 + c) * GT] = floatx4{acc[i][j][4 * c], acc[i][j][4 * c + 1], acc[i][j][4 * c + 2], acc[i][j][4 * c + 3]};
        if (zero_points && lane == 0) atomicOr(a.zflags + t, 1u);
        return;
    }
    if (zero_points) {
        // (columns past N read clamped rows and may trigger this needlessly; nothing is stored for them)
        {
            // first the cheap way: at most eight columns with zero-points, strips in this wavefront's own
            // corner of the weight ring (its copies have landed; nobody else touches it)
            const uint32_t strips = lds_base + kWRingBase + (uint32_t)wave * 1024u;
            StripColumns cols;
            if (zero_point_terms_few_columns(a, n0 + wn * 64, m0, lane, strips, cols)) {
#pragma unroll
                for (int i = 0; i < 4; ++i) store_rows<2>(a, acc[i], m0 + 32 * i, n0, wn, lane, 32 * i, strips, &cols);
                return;
            }
        }
        // otherwise a table of all 64 columns, 32 rows at a time, in the activation ring (which does not
        // overlap any wavefront's strips) -- once all four wavefronts have drained their copies and left
        // the main loop
        static_assert(kWStageBytes == 4096 && kWStages * 2 >= kStrips, "two strips of 128 floats in the wavefront's KiB of every stage");
        static_assert(4 * 32 * 64 * 4 <= kWRingBase, "four tables of 32 x 64 floats inside the activation ring");
        const uint32_t table = lds_base + (uint32_t)wave * (32 * 64 * 4);
        while (__builtin_amdgcn_readfirstlane((int)lds_read_f32_bits_now(lds_base + kDoneWord)) != GT / kWave) __builtin_amdgcn_s_sleep(2);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            zero_point_terms<32>(a, n0 + wn * 64, m0 + 32 * i, lane, table);
            store_rows<1>(a, acc[i], m0 + 32 * i, n0, wn, lane, 0, table);
        }
        return;
    }
    store_tile(a, acc, m0, n0, wn, lane);
}

// Second launch of a split-K matmul: four workgroups per tile, one per 32-row slab, add the shares
// in split order (thread and register layout as in the contraction kernel) and finish the slab.
__global__ __launch_bounds__(GT) void gemm_reduce_kernel(const GemmArgs a, int tiles_m, int tiles_n) {
    const int t = (int)(blockIdx.x >> 2), i = (int)(blockIdx.x & 3), tid = threadIdx.x, lane = tid & 63, wn = tid >> 6;
    int tm, tn;
    tile_coords(t, tiles_m, tiles_n, tm, tn);
    const floatx4* const all = reinterpret_cast<const floatx4*>(a.partial) + ((int64_t)t * a.splits * 32) * GT + tid;
    floatx16 acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int piece = (i * 2 + j) * 4 + c;
            floatx4 share[kGemmMaxSplits];  // all loads first (absent splits re-read share 0), then the sum in split order
#pragma unroll
            for (int sp = 0; sp < kGemmMaxSplits; ++sp) share[sp] = all[((int64_t)(sp < a.splits ? sp : 0) * 32 + piece) * GT];
            floatx4 sum = share[0];
#pragma unroll
            for (int sp = 1; sp < kGemmMaxSplits; ++sp)
                if (sp < a.splits) sum = sum + share[sp];
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[j][4 * c + e] = sum[e];
        }
    const int64_t m_first = (int64_t)tm * GM + i * 32, n0 = (int64_t)tn * GN;
    if (a.zflags[t] != 0u) {
        __shared__ __align__(16) float tables[4 * 32 * 64];  // one per wavefront
        const uint32_t table = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) float*)tables + (uint32_t)wn * (32 * 64 * 4);
        zero_point_terms<32>(a, n0 + wn * 64, m_first, lane, table);
        store_rows<1>(a, acc, m_first, n0, wn, lane, 0, table);
        return;
    }
    store_rows<0>(a, acc, m_first, n0, wn, lane);
}

// Splits of K per tile: when the tiles alone leave three quarters of the chip idle, enough workgroups
// for its 512 slots (two per compute unit), each split at least four blocks long.  A function of the
// shape only.
int gemm_splits(int64_t M, int64_t N, int64_t K) {
    const int64_t tiles = ((M + GM - 1) / GM) * ((N + GN - 1) / GN);
    if (tiles > kGemmSplitMaxTiles) return 1;
    int64_t s = 512 / tiles;
    if (s > kGemmMaxSplits) s = kGemmMaxSplits;
    if (s > K / kBlock / 4) s = K / kBlock / 4;
    return s < 1 ? 1 : (int)s;
}
size_t gemm_partial_bytes(int64_t M, int64_t N, int64_t K) {
    const int s = gemm_splits(M, N, K);
    return s > 1 ? (size_t)s * (size_t)(((M + GM - 1) / GM) * ((N + GN - 1) / GN)) * (GM * GN * 4) : 0;
}

int launch_gemm(const uint32_t* codes, const uint32_t* scales, int64_t N, int64_t K, const _Float16* Xt, const _Float16* X, int64_t ldx,
                int64_t M, void* Y, int y_f16, int64_t ldy, float* partial, size_t partial_bytes, uint32_t* zflags, uint32_t* flags,
                hipStream_t stream) {
    GemmArgs a;
    a.codes = codes; a.scales = scales; a.Xt = Xt; a.X = X; a.ldx = ldx; a.Y = Y; a.flags = flags;
    a.N = N; a.K = K; a.M = M; a.ldy = ldy; a.NT = (int)((N + 15) / 16); a.KB = (int)(K / kBlock); a.y_f16 = y_f16;
    a.partial = partial; a.zflags = zflags;
    // split only if the caller's workspace has room for the shares (a grouped call sizes it for its largest tensor)
    a.splits = partial != nullptr && zflags != nullptr && gemm_partial_bytes(M, N, K) <= partial_bytes ? gemm_splits(M, N, K) : 1;
    const LaunchTiming tm = take_launch_timing();
    const int64_t tiles_m = (M + GM - 1) / GM, tiles_n = (N + GN - 1) / GN;
    if (K > kGemmMaxK || tiles_m * tiles_n >= 0x7fffffff / 8 / kGemmMaxSplits) return -2;
    const int per = (int)((tiles_m * tiles_n * a.splits + 7) / 8);
    const dim3 g((unsigned)(per * 8));
    static std::atomic<bool> lds_limit_raised{false};
    if (!lds_limit_raised) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds) != hipSuccess) return -6;
        lds_limit_raised = true;
    }
    if (tm.start != nullptr) hipExtLaunchKernelGGL(gemm_kernel, g, dim3(GT), kGemmLds, stream, tm.start, tm.stop, 0, a, (int)tiles_m, (int)tiles_n, per);
    else hipLaunchKernelGGL(gemm_kernel, g, dim3(GT), kGemmLds, stream, a, (int)tiles_m, (int)tiles_n, per);
    if (hipGetLastError() != hipSuccess) return -6;
    if (a.splits > 1) {
        hipLaunchKernelGGL(gemm_reduce_kernel, dim3((unsigned)(tiles_m * tiles_n * 4)), dim3(GT), 0, stream, a, (int)tiles_m, (int)tiles_n);
        if (hipGetLastError() != hipSuccess) return -6;
    }
    return 0;
}

}  // namespace itq3s
