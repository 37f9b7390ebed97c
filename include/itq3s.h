/*
 * libitq3s -- ITQ3_S fused 3-bit ternary matmul for AMD MI355X (gfx950).  C ABI.
 *
 * ITQ3_S (arxiv 2603.27914) stores a weight matrix W[N,K] in blocks of 256 consecutive input
 * channels of one output row.  Each block is rotated by the normalised 256-point Walsh-Hadamard
 * transform H, scaled, and coded with ternary digits; 256 three-bit codes + fp16 scale d + fp16
 * zero-point z = 100 bytes (Sec. 4.1).  Reconstruction is w_hat = H( d (q - z) ) (Prop. 1).
 *
 * Conventions for every call below
 *   - all data pointers are DEVICE pointers owned by the caller; the calls declared in this header
 *     never allocate, free or synchronise.  Work is enqueued on `stream` (a hipStream_t passed as
 *     void*; NULL = the default stream) and the call returns at once.
 *   - the return value is 0 (ITQ3S_OK) or a negative ITQ3S_ERR_* code.  Argument errors are found
 *     on the host before anything is launched; then no kernel runs and no memory is touched.
 *   - `status_flags` (may be NULL) is one device uint32 into which kernels OR data-condition bits
 *     (ITQ3S_FLAG_*); the caller clears and reads it.
 *   - calls may come from several host threads at once: the library keeps no mutable state apart
 *     from cached device properties.  Calls that share a workspace or an output must be ordered by
 *     the caller (same stream, or events).
 *   - K must be a multiple of 256 (the paper leaves other widths open, Sec. 8).  N is arbitrary;
 *     storage is padded to a multiple of 16 rows.
 *
 * Packed layout (Sec. 4.1-4.2; the paper's word formula is not self-consistent, the bit positions
 * are this library's choice within the 96 + 2 + 2 byte budget):
 *   KB = K/256, NT = ceil(N/16).  Tile (nt, b) = rows 16nt..16nt+15 x channels 256b..256b+255,
 *   stored at index nt*KB + b.
 *   codes : NT*KB tiles of 384 little-endian uint32 (1536 bytes = 16 blocks x 96 bytes).
 *           For element e (0..255) of tile row r (0..15), code c = q+1 in {0,1,2}:
 *             lane = 16*(e>>6) + r,  i = e & 63
 *             low plane  word 4*lane + (i>>4),       bits [2(i&15)+1 : 2(i&15)] = c & 3
 *             high plane word 256 + 2*lane + (i>>5), bit  (i&31)                = c >> 2  (0 on encode)
 *           i.e. wavefront lane `lane` finds its 64 codes in one 16-byte and one 8-byte load, laid
 *           out as the 16x16xK MFMA operand of row r.
 *   scales: NT*KB*16 uint32; word (nt*KB + b)*16 + r = fp16 bits of d | fp16 bits of z << 16.
 *   Rows >= N of the last tile hold code 1 and scale word 0.
 */
#ifndef ITQ3S_H
#define ITQ3S_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ITQ3S_OK 0
#define ITQ3S_ERR_NULL (-1)      /* a required pointer is NULL                                    */
#define ITQ3S_ERR_SHAPE (-2)     /* N, K, M <= 0, K % 256 != 0, or a leading dimension too small   */
#define ITQ3S_ERR_ALIGN (-3)     /* a pointer or leading dimension breaks the stated alignment     */
#define ITQ3S_ERR_DTYPE (-4)     /* dtype argument is not ITQ3S_F32 / ITQ3S_F16                    */
#define ITQ3S_ERR_WORKSPACE (-5) /* workspace NULL or smaller than itq3s_matmul_workspace_bytes    */
#define ITQ3S_ERR_LAUNCH (-6)    /* the HIP runtime refused a launch (see hipGetLastError)         */

#define ITQ3S_F32 0
#define ITQ3S_F16 1

#define ITQ3S_FLAG_NONFINITE 1u /* quantize: a weight was NaN/Inf; its block is stored as zeros    */
#define ITQ3S_FLAG_SCALE_SAT 2u /* quantize: d exceeded the fp16 range and was clamped to 65504    */
#define ITQ3S_FLAG_Z_CLAMP 4u   /* quantize: |z| exceeded 2048 and was clamped                     */
#define ITQ3S_FLAG_BAD_CODE 8u  /* decode: a code outside {0,1,2} was met (dequantize checks both
                                   planes; matmul checks the high plane only and treats a low-plane
                                   3 as digit +2)                                                  */
#define ITQ3S_FLAG_ACT_RANGE 16u /* matmul: a rotated activation left the fp16 range (see itq3s_matmul);
                                   the outputs that depend on that 256-channel chunk are Inf or NaN */

/* Sizes of the two packed arrays for W[N,K]: NT*KB*1536 and NT*KB*64 bytes (0 if K % 256 != 0). */
size_t itq3s_codes_bytes(int64_t N, int64_t K);
size_t itq3s_scales_bytes(int64_t N, int64_t K);

/* Bytes of scratch itq3s_matmul needs (Sec. 2.3: H is symmetric and its own inverse, so
 * <H v, x> = <v, H x>; the library rotates X once per call instead of every weight block).  Never 0.
 * M <= 4: 256 (the streaming kernel rotates inside the kernel; the workspace is not touched).
 * Larger M: room for the rotated activations, grows with M*K; for M > 16 and shapes with few output
 * tiles (at most 128 tiles of 128 x 256) also the partial sums of the workgroups that share a tile's
 * K range (up to 8 x M x N x 4 bytes, tiles rounded up).  A function of the three sizes only. */
size_t itq3s_matmul_workspace_bytes(int64_t M, int64_t N, int64_t K);

/* Offline quantization (Alg. 1, Def. 1).  Per block: w' = H w in fp64 (butterfly stages
 * 1,2,4,...,128, then x 1/16); d = 0.7979 * population-std(w') rounded to fp16 through fp32;
 * z = -floor(mean(w')/d + 0.5); code = 1 + clamp(floor(w'/d + z + 0.5), -1, 1), decided exactly
 * through the thresholds (+-0.5 - z) d.  Sums are pairwise (neighbours first).  Results are
 * bit-identical on any IEEE-754 machine.
 *   W      [in]  device, N x K fp32 row-major, row stride ldw elements (ldw >= K, ldw % 4 == 0,
 *                pointer 16-byte aligned)
 *   codes  [out] device, itq3s_codes_bytes(N,K), 16-byte aligned
 *   scales [out] device, itq3s_scales_bytes(N,K), 16-byte aligned */
int itq3s_quantize(const float *W, int64_t N, int64_t K, int64_t ldw, uint32_t *codes, uint32_t *scales,
                   uint32_t *status_flags, void *stream);

/* Weight-side reconstruction (Alg. 2, Prop. 1): W_out[n][k] = ( H( d (q - z) ) )[k], computed with
 * exact integer butterflies and one rounding to the output type.
 *   W_out [out] device, N x K of out_dtype (ITQ3S_F32 or ITQ3S_F16), row stride ldo elements
 *               (ldo >= K, ldo % 4 == 0, pointer 16-byte aligned) */
int itq3s_dequantize(const uint32_t *codes, const uint32_t *scales, int64_t N, int64_t K, void *W_out, int out_dtype,
                     int64_t ldo, uint32_t *status_flags, void *stream);

/* Fused matmul (problem statement of Alg. 2; Sec. 5.4 for M = 1):  Y[m][n] = sum_k X[m][k] w_hat[n][k].
 * No dequantized weight is written to memory.  M <= 16 takes the bandwidth-bound streaming path
 * (M <= 32: two passes of it), larger M the tiled MFMA path (which accepts K <= 4194304 only:
 * ITQ3S_ERR_SHAPE beyond; the streaming path K <= 2^28); fp32 accumulation in both, the zero-point
 * terms included: an output element is rounded once.
 * Activation range.  Every 256-channel chunk x of a row of X is replaced by x~ = H x, rounded to
 * fp16, after an intermediate T = X_16x16 H_16 / 4 that is split into fp16 parts.  Both stay
 * finite whenever  max|x| <= 16376  and  |(H x)_k| <= 65504  over the chunk (the second holds if
 * sum|x| <= 16 * 65504; any chunk with max|x| <= 4094 satisfies both).  Outside that range the
 * products that involve the chunk are Inf/NaN although the exact result is finite, and
 * ITQ3S_FLAG_ACT_RANGE is OR-ed into status_flags.  Scale such activations down by a power of
 * two (the product is linear) before the call.
 *   X  [in]  device, M x K fp16 row-major, row stride ldx elements (ldx >= K, ldx % 8 == 0,
 *            pointer 16-byte aligned)
 *   Y  [out] device, M x N of y_dtype, row stride ldy elements (ldy >= N); overwritten
 *   workspace [scratch] device, 256-byte aligned, at least itq3s_matmul_workspace_bytes(M,N,K);
 *            contents undefined afterwards; calls sharing a workspace must be stream-ordered */
int itq3s_matmul(const uint32_t *codes, const uint32_t *scales, int64_t N, int64_t K, const void *X, int64_t M, int64_t ldx,
                 void *Y, int y_dtype, int64_t ldy, void *workspace, size_t workspace_bytes, uint32_t *status_flags,
                 void *stream);

/* itq3s_matmul for callers that cannot hand over a workspace because they cannot allocate device
 * memory: code that runs under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same kernels and bit-identical results; the scratch memory is a
 * library-owned static device array of ITQ3S_STATIC_SCRATCH_BYTES (every GPU the library runs on
 * holds one until the process ends), and the call allocates nothing.
 *   - returns ITQ3S_ERR_WORKSPACE without launching anything if
 *     itq3s_matmul_workspace_bytes(M, N, K) > ITQ3S_STATIC_SCRATCH_BYTES (M <= 4 always fits);
 *   - all calls on one GPU share that array, which keeps the last call's contents: calls that overlap
 *     in time on one GPU (two streams, two threads) race and must be ordered by the caller;
 *   - the first call on a device looks up the array's address (no allocation, no synchronisation). */
#define ITQ3S_STATIC_SCRATCH_BYTES (64u << 20)
int itq3s_matmul_static(const uint32_t *codes, const uint32_t *scales, int64_t N, int64_t K, const void *X, int64_t M,
                        int64_t ldx, void *Y, int y_dtype, int64_t ldy, uint32_t *status_flags, void *stream);

/* Several weight tensors with the same K against the same activations in ONE call: Y_t = X W_hat_t^T
 * for t = 0..count-1 (1 <= count <= ITQ3S_MAX_GROUP), e.g. the query/key/value projections of a layer,
 * or gate and up.  For M <= 16 all tensors are served by a single launch of the streaming kernel, so
 * the launch latency and the ramp of the memory pipeline are paid once; for larger M the activations
 * are rotated once and one tiled launch per tensor follows.  Results are identical to count calls of
 * itq3s_matmul.
 *   w  [in] HOST array of count descriptors (read during the call, not kept): device pointers codes,
 *           scales (as for itq3s_matmul), rows N, output Y (M x N of y_dtype, row stride ldy >= N)
 *   X, M, ldx, y_dtype, status_flags, stream: as for itq3s_matmul
 *   workspace: at least the largest itq3s_matmul_workspace_bytes(M, N_t, K) over the tensors of the call
 *           (ITQ3S_ERR_WORKSPACE otherwise: how a tensor is computed never depends on the room given) */
#define ITQ3S_MAX_GROUP 4
typedef struct itq3s_weight {
    const uint32_t *codes;
    const uint32_t *scales;
    int64_t N;
    void *Y;
    int64_t ldy;
} itq3s_weight;
int itq3s_matmul_grouped(const itq3s_weight *w, int count, int64_t K, const void *X, int64_t M, int64_t ldx, int y_dtype,
                         void *workspace, size_t workspace_bytes, uint32_t *status_flags, void *stream);

/* The same product with the rotation on the WEIGHT side, the way the paper's kernel does it (Alg. 2):
 * every 256-channel block of a weight tile is unpacked, scaled and passed through the inverse
 * transform on its way into on-chip memory, then multiplied with the un-rotated activations on the
 * matrix cores; no dequantized weight is written to memory and no workspace is needed.  Results
 * agree with itq3s_matmul within the same tolerance (the rounding sits on w_hat instead of H x).  A
 * reconstructed 128-row weight tile is shared by 512 rows of X, so the transform of the whole tensor
 * is repeated ceil(M/512) times; the call is meant for comparing the two placements, not as the fast
 * path.  Arguments as for itq3s_matmul; any M with ceil(M/512) <= 65535.
 * (A variant that also reports the kernel's duration is declared in itq3s_bench.h.) */
int itq3s_matmul_weight_side(const uint32_t *codes, const uint32_t *scales, int64_t N, int64_t K, const void *X, int64_t M,
                             int64_t ldx, void *Y, int y_dtype, int64_t ldy, uint32_t *status_flags, void *stream);

/* Block-size ablation (Sec. 6, "Ablation: FWHT Block Size"): rotate, quantize and reconstruct with a
 * transform length block_size in {32, 64, 128, 256, 512} instead of the format's 256, without
 * packing.  Per block of block_size consecutive channels of a row the steps are those of
 * itq3s_quantize (fp64, fixed order, 1/sqrt(block_size) applied once after the butterflies, scale
 * rounded to fp16, zero-point, exact thresholds) followed by w_hat = H(d (q - z)) (Alg. 2, Prop. 1),
 * rounded once to fp32.  With block_size 256 the codes and scale words equal what itq3s_quantize
 * packs and w_hat agrees with itq3s_dequantize's fp32 output.
 *   W (device, const): N x K fp32, row stride ldw >= K, ldw % 4 == 0, 16-byte aligned
 *   K % block_size == 0
 *   codes_out (device, may be NULL): N x K bytes, one code 0/1/2 per channel, 16-byte aligned
 *   scales_out (device, may be NULL): N x (K / block_size) words, d | z << 16 as in the packed format
 *   W_hat (device, may be NULL): N x K fp32, row stride ldo >= K, ldo % 4 == 0, 16-byte aligned
 *   err2 (device, may be NULL): two doubles the call ADDS to (zero them first): [0] += sum (w_hat - w)^2,
 *       [1] += sum w^2 over all blocks without non-finite weights.  The additions are atomic and
 *       their order is not fixed: the sums are reproducible to rounding only.
 *   status_flags: as for itq3s_quantize
 * Blocks with a non-finite weight or a zero scale give codes 1, scale word 0, w_hat 0.
 * Returns ITQ3S_ERR_SHAPE for any other block_size. */
int itq3s_roundtrip(const float *W, int64_t N, int64_t K, int64_t ldw, int block_size, uint8_t *codes_out, uint32_t *scales_out,
                    float *W_hat, int64_t ldo, double *err2, uint32_t *status_flags, void *stream);

/* ---- The sub-block-scale variant of the format (Sec. 4.1, "Block Structure": 8 fp16 sub-block scales
 * for 8 sub-blocks of 32 elements, 116 bytes per block, 3.625 bit/weight).  The paper names the option
 * and its size and gives no formula; this library's reading:
 *   - sub-block j = rotated coefficients 32j .. 32j+31 of the block (the domain the codes live in);
 *   - d and z are exactly those of the 100-byte format (codes and scales arrays keep their layout and
 *     meaning; the zero-point stays in units of d);
 *   - s_j = 0.7979 sigma_j / d, sigma_j the deviation of the sub-block's coefficients about the block
 *     mean, rounded to fp16 through fp32 (the rule of Sec. 3.3 applied per sub-block);
 *   - code = 1 + clamp(floor((w'/d + z) / s_j + 0.5), -1, 1)  (Def. 1 with the digit step s_j);
 *   - w_hat = H( d (s_j q - z) )  (Prop. 1 with the scaled digit).
 * With every s_j = 1 this is the 100-byte format.
 *   subscales: NT*KB*64 uint32 (itq3s_subscales_bytes), 16-byte aligned; word (nt*KB + b)*64 + 16 g + r =
 *     fp16 s_(2g) | fp16 s_(2g+1) << 16 for tile row r and quarter g of the block (0 for rows >= N).
 * Other arguments, flags and errors as for itq3s_quantize / itq3s_dequantize / itq3s_matmul.
 * itq3s_matmul_sub: up to M = 64 it runs ceil(M/16) passes of the streaming kernel, above that the
 * tiled kernel that reconstructs weight tiles on chip (the placement of itq3s_matmul_weight_side; one
 * pass over the weights per 512 rows, ceil(M/512) <= 65535).  workspace: for 5 <= M <= 64 at least
 * itq3s_matmul_workspace_bytes(min(M, 16), N, K) bytes, 256-byte aligned (the rotated activations of a
 * pass), else ITQ3S_ERR_WORKSPACE; not used for other M (may be NULL).  The
 * streaming kernel multiplies with the sub-scales in fp16: exact for 1/16 <= s_j <= 4094 (the
 * quantizer's values lie below 3); smaller ones lose low bits of a small contribution, larger ones
 * are not supported. */
size_t itq3s_subscales_bytes(int64_t N, int64_t K);
int itq3s_quantize_sub(const float *W, int64_t N, int64_t K, int64_t ldw, uint32_t *codes, uint32_t *scales,
                       uint32_t *subscales, uint32_t *status_flags, void *stream);
int itq3s_dequantize_sub(const uint32_t *codes, const uint32_t *scales, const uint32_t *subscales, int64_t N, int64_t K,
                         void *W_out, int out_dtype, int64_t ldo, uint32_t *status_flags, void *stream);
int itq3s_matmul_sub(const uint32_t *codes, const uint32_t *scales, const uint32_t *subscales, int64_t N, int64_t K,
                     const void *X, int64_t M, int64_t ldx, void *Y, int y_dtype, int64_t ldy, void *workspace,
                     size_t workspace_bytes, uint32_t *status_flags, void *stream);

/* Static text for a status code.  Never NULL. */
const char *itq3s_strerror(int status);

/* major*10000 + minor*100 + patch */
int itq3s_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ITQ3S_H */
