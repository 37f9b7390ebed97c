// Internal launch interface between the C-ABI entry points and the kernels.  Every launcher
// assumes arguments were validated by the caller, enqueues on `stream` and returns 0 or -6.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace itq3s {

constexpr uint32_t kFlagNonFinite = 1u, kFlagScaleSat = 2u, kFlagZClamp = 4u, kFlagBadCode = 8u, kFlagActRange = 16u;

// Streaming path handles up to this many activation rows; more rows go to the tiled MFMA path.
constexpr int kGemvMaxM = 16;
// Up to this many rows the streaming kernel rotates the activations itself (one launch, no workspace).
constexpr int kGemvFusedMaxM = 4;
// One streaming launch serves up to this many weight tensors that share K and the activations.
constexpr int kGemvMaxGroup = 4;

// Optional device-side timing of the contraction kernel.  set_launch_timing() arms a pair of events;
// the next launch of a contraction kernel (streaming or tiled) takes them (take_launch_timing clears
// the pair) and attaches them to its own dispatch, so that their distance is the kernel's duration
// by the GPU's timestamps, without launch gaps.  Not thread-safe: a measurement aid.
struct LaunchTiming {
    hipEvent_t start = nullptr, stop = nullptr;
};
void set_launch_timing(hipEvent_t start, hipEvent_t stop);
LaunchTiming take_launch_timing();

// subscales: null for the 100-byte format; the sub-scale array of the 116-byte variant otherwise
// (64 words per tile: word 16 g + r = fp16 s_2g | fp16 s_(2g+1) << 16 for tile row r, quarter g).
int launch_quantize(const float* W, int64_t N, int64_t K, int64_t ldw, uint32_t* codes, uint32_t* scales, uint32_t* subscales, uint32_t* flags,
                    hipStream_t stream);

int launch_dequantize(const uint32_t* codes, const uint32_t* scales, const uint32_t* subscales, int64_t N, int64_t K, void* out, int out_f16,
                      int64_t ldo, uint32_t* flags, hipStream_t stream);

// Rotated activations for the streaming path with 5..16 rows: Xt in MFMA operand order with MP (8 or
// 16) columns; S[b*MP + m] = sum over the rounded rotated chunk, S[KB*MP + b*MP + m] = the exact
// sum of the unrounded one, 16 x[m][256 b].  flags (may be null): kFlagActRange is OR-ed in if a
// rotated value leaves the fp16 range.
int launch_rotate_frag(const _Float16* X, int64_t M, int64_t K, int64_t ldx, int MP, _Float16* Xt, float* S, uint32_t* flags, hipStream_t stream);

// Rotated activations for the tiled path: Xt[m][k] row-major, row stride K.
// (also clears n_zero words at zero_words: the split-K flags of the contraction that follows)
int launch_rotate_rowmajor(const _Float16* X, int64_t M, int64_t K, int64_t ldx, _Float16* Xt, uint32_t* zero_words, int n_zero, uint32_t* flags,
                           hipStream_t stream);

// One weight tensor of a streaming launch and where its product goes.
struct GemvWeight {
    const uint32_t* codes;
    const uint32_t* scales;
    int64_t N;
    void* Y;
    int64_t ldy;
    const uint32_t* subscales = nullptr;  // the 116-byte variant's sub-scales (then the launch takes this one tensor only)
};

// count (1..kGemvMaxGroup) tensors W_t[N_t, K] against the same activations X[M][ldx], M <= kGemvFusedMaxM,
// in one launch that rotates the activations itself.
int launch_gemv(const GemvWeight* w, int count, int64_t K, const _Float16* X, int64_t ldx, int64_t M, int y_f16, uint32_t* flags,
                hipStream_t stream);

// The same for kGemvFusedMaxM < M <= kGemvMaxM: Xt = rotated activations in operand order with MP
// columns and S = their block sums, both from launch_rotate_frag.
int launch_gemv_rows(const GemvWeight* w, int count, int64_t K, const _Float16* Xt, const float* S, int64_t M, int MP, int y_f16,
                     uint32_t* flags, hipStream_t stream);

// Compute units of the current device (cached).
int cu_count();

// Tiled matmul, M > 16.  Xt = rotated activations (launch_rotate_rowmajor); X, ldx = the activations
// themselves (zero-point term).  Shapes with few output tiles split K over several workgroups per tile
// and add the shares in a second launch (gemm_splits > 1): those use `partial` (gemm_partial_bytes,
// 16-byte aligned; partial_bytes = what is there -- too little, or none, means no split) and
// `zflags` (kGemmFlagWords words, all zero at launch).
constexpr int kGemmMaxSplits = 8;
constexpr int kGemmSplitMaxTiles = 128;  // more tiles than this: no split
constexpr int kGemmFlagWords = 128;
int gemm_splits(int64_t M, int64_t N, int64_t K);
size_t gemm_partial_bytes(int64_t M, int64_t N, int64_t K);
int launch_gemm(const uint32_t* codes, const uint32_t* scales, int64_t N, int64_t K, const _Float16* Xt, const _Float16* X, int64_t ldx,
                int64_t M, void* Y, int y_f16, int64_t ldy, float* partial, size_t partial_bytes, uint32_t* zflags, uint32_t* flags,
                hipStream_t stream);

// Tiled matmul with the inverse transform applied to the weights inside the tile loader (Alg. 2 as
// printed); X = the activations themselves.  Any M.  subscales: the 116-byte variant's array, or null.
int launch_gemm_weight_side(const uint32_t* codes, const uint32_t* scales, const uint32_t* subscales, int64_t N, int64_t K, const _Float16* X,
                            int64_t ldx, int64_t M, void* Y, int y_f16, int64_t ldy, uint32_t* flags, hipStream_t stream);

// Round trip with transform length n in {32 .. 512} (block-size ablation, Sec. 6); any of codes,
// scales, What, err may be null.  Returns -2 for another n.
int launch_roundtrip(const float* W, int64_t N, int64_t K, int64_t ldw, int n, uint8_t* codes, uint32_t* scales, float* What, int64_t ldo,
                     double* err, uint32_t* flags, hipStream_t stream);

}  // namespace itq3s
