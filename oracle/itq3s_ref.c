/*
 * ITQ3_S reference oracle: plain, slow, single-threaded CPU code in fp64.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the smoke check and
 * the benchmark's cpu_baseline leg may call it.  It shares no source, header, table or helper
 * with the HIP library; each side implements the storage format from its written description.
 *
 * Every function follows one passage of the paper (arxiv 2603.27914) and says which.  Where the
 * paper is silent, garbled or at odds with itself the reading taken is stated next to the code.
 *
 * Build:  gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC itq3s_ref.c -o libitq3s_ref.so -lm
 * (contraction is switched off so that every fp64 operation rounds once, as written.)
 *
 * ---------------------------------------------------------------------------------------------
 * Storage format (Sec. 4.1 "Block Structure", Sec. 4.2 "Interleaved Packing"):
 *   A block is 256 consecutive input channels k of one output row n.  Per block: 256 codes of
 *   3 bits (96 bytes) + fp16 scale d_k + fp16 zero-point z_k = 100 bytes (3.125 bit/weight).
 *   A code is c = q + 1 in {0,1,2} for the ternary digit q in {-1,0,+1} (Sec. 4.2, first sentence).
 *   The low two bits of c ("q mod 4" in the packing equation) and its high bit are kept in two
 *   bit-planes; the high bit is always 0 on encode.  The paper's word-level formula is
 *   self-contradictory (8 nibbles per word would be 128 bytes, not 96) and it prints no example,
 *   so the bit positions below are this library's own choice, fixed only by the 96-byte budget:
 *
 *   Blocks are grouped in tiles of 16 rows x 1 block column.  Tile (nt, b) covers rows
 *   16*nt .. 16*nt+15 and channels 256*b .. 256*b+255; tiles are stored in order nt*KB + b
 *   (KB = K/256), 384 little-endian uint32 each (16 blocks x 96 bytes):
 *     element e (0..255) of row r (0..15) of the tile:   lane = 16*(e>>6) + r,  i = e & 63
 *       low plane : word 4*lane + (i>>4),        bits [2*(i&15)+1 : 2*(i&15)]  = c & 3
 *       high plane: word 256 + 2*lane + (i>>5),  bit  (i&31)                   = c >> 2
 *   The scales array holds one uint32 per block at index (nt*KB + b)*16 + r:
 *     bits 0..15 = fp16 d_k, bits 16..31 = fp16 z_k.
 *   Rows past N in the last tile are stored as code 1 (digit 0) with scale word 0.
 * ---------------------------------------------------------------------------------------------
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ITQ3S_REF_BLOCK 256
#define ITQ3S_REF_TILE_ROWS 16
#define ITQ3S_REF_TILE_WORDS 384

/* Optimal-ternary-scale constant: the paper prints it as 0.798 (Sec. 3.3) and as t* ~ 0.7979
 * (App. A).  Its closed form as printed does not evaluate to that number, so the decimal the
 * paper prints with most digits is taken literally. */
static const double ITQ3S_REF_T_STAR = 0.7979;

/* data-condition flags OR-ed into *flags (may be NULL) */
#define REF_FLAG_NONFINITE 1u      /* a weight was NaN/Inf: block stored as all-zero            */
#define REF_FLAG_SCALE_SAT 2u      /* d_k exceeded the fp16 range and was clamped to 65504        */
#define REF_FLAG_Z_CLAMP 4u        /* |z_k| exceeded 2048 and was clamped                         */
#define REF_FLAG_BAD_CODE 8u       /* decode met a code outside {0,1,2}                           */

/* ------------------------------------------------------------------ fp16 <-> fp32, bit level */

/* fp32 -> fp16 bits, round to nearest even, overflow to infinity, gradual underflow. */
static uint16_t ref_f32_to_f16(float f)
{
    uint32_t x;
    memcpy(&x, &f, 4);
    uint32_t sign = (x >> 16) & 0x8000u;
    uint32_t ex = (x >> 23) & 0xffu;
    uint32_t man = x & 0x7fffffu;
    if (ex == 0xffu) return (uint16_t)(sign | 0x7c00u | (man ? 0x200u : 0u));
    int e = (int)ex - 127 + 15;
    if (e >= 31) return (uint16_t)(sign | 0x7c00u);
    if (e <= 0) {
        if (e < -10) return (uint16_t)sign;            /* below half of the smallest subnormal */
        man |= 0x800000u;                               /* make the leading 1 explicit          */
        int shift = 14 - e;                             /* 14..24                               */
        uint32_t kept = man >> shift;
        uint32_t rem = man & ((1u << shift) - 1u);
        uint32_t half = 1u << (shift - 1);
        if (rem > half || (rem == half && (kept & 1u))) kept++;
        return (uint16_t)(sign | kept);
    }
    uint32_t kept = man >> 13;
    uint32_t rem = man & 0x1fffu;
    uint32_t out = ((uint32_t)e << 10) | kept;
    if (rem > 0x1000u || (rem == 0x1000u && (kept & 1u))) out++;   /* carry may bump exponent */
    return (uint16_t)(sign | out);
}

static double ref_f16_to_f64(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int ex = (h >> 10) & 0x1f;
    int man = h & 0x3ff;
    double v;
    if (ex == 0) v = ldexp((double)man, -24);
    else if (ex == 31) v = man ? NAN : INFINITY;
    else v = ldexp((double)(man | 0x400), ex - 25);
    return sign ? -v : v;
}

/* ------------------------------------------------------------------ transform and sums */

/* Unnormalised 256-point Walsh-Hadamard butterfly network (Sec. 2.3 butterfly equation; stage
 * order and pairing as in Alg. 2 / App. B: step = 1,2,4,...,128, partner index = i XOR step, the
 * lower index receives u+v and the higher one u-v).  In place. */
void itq3s_ref_fwht256(double *a)
{
    for (int step = 1; step < ITQ3S_REF_BLOCK; step <<= 1)
        for (int i = 0; i < ITQ3S_REF_BLOCK; i++)
            if ((i & step) == 0) {
                double u = a[i], v = a[i + step];
                a[i] = u + v;
                a[i + step] = u - v;
            }
}

/* Sum of 256 values by pairwise halving: neighbours first (distance 1), then distance 2, ...
 * The shape is fixed so that any machine adding the same pairs gets the same bits. */
static double ref_pairwise_sum256(const double *v)
{
    double t[ITQ3S_REF_BLOCK];
    memcpy(t, v, sizeof t);
    for (int step = 1; step < ITQ3S_REF_BLOCK; step <<= 1)
        for (int i = 0; i < ITQ3S_REF_BLOCK; i += 2 * step) t[i] = t[i] + t[i + step];
    return t[0];
}

/* ------------------------------------------------------------------ format addressing */

static inline size_t ref_tile_index(int64_t n, int64_t b, int64_t KB) { return (size_t)((n >> 4) * KB + b); }

static void ref_put_code(uint32_t *tile, int r, int e, uint32_t c)
{
    int lane = 16 * (e >> 6) + r, i = e & 63;
    uint32_t *lo = &tile[4 * lane + (i >> 4)];
    uint32_t *hi = &tile[256 + 2 * lane + (i >> 5)];
    int sh = 2 * (i & 15);
    *lo = (*lo & ~(3u << sh)) | ((c & 3u) << sh);
    *hi = (*hi & ~(1u << (i & 31))) | (((c >> 2) & 1u) << (i & 31));
}

static uint32_t ref_get_code(const uint32_t *tile, int r, int e)
{
    int lane = 16 * (e >> 6) + r, i = e & 63;
    uint32_t lo = (tile[4 * lane + (i >> 4)] >> (2 * (i & 15))) & 3u;
    uint32_t hi = (tile[256 + 2 * lane + (i >> 5)] >> (i & 31)) & 1u;
    return lo | (hi << 2);
}

size_t itq3s_ref_codes_bytes(int64_t N, int64_t K) { return (size_t)((N + 15) / 16) * (size_t)(K / 256) * 1536u; }
size_t itq3s_ref_scales_bytes(int64_t N, int64_t K) { return (size_t)((N + 15) / 16) * (size_t)(K / 256) * 64u; }

/* ------------------------------------------------------------------ quantize (Alg. 1, Def. 1) */

/* One block.  w: 256 fp32 weights.  codes_out: 256 codes in {0,1,2}.  Returns the scale word.
 *
 * Steps, in the order of Alg. 1:
 *   w'  = H w                         (normalised transform: butterflies, then x 1/16)
 *   d_k = T* . sigma(w')              (the algorithm's fraction is dimensionally wrong as printed;
 *                                      Sec. 3.3 says the scale is T* times the empirical standard
 *                                      deviation of the transformed block.  sigma is the population
 *                                      deviation about the mean, both over 256)
 *   d_k is rounded to fp16 (via fp32, both steps to nearest even) BEFORE coding, so that encoder
 *   and decoder see the same grid.
 *   z_k = -round(mu(w') / d_k)        (round = floor(x + 0.5), as in Def. 1)
 *   q   = clamp(floor(w'/d_k + z_k + 0.5), -1, 1)            (Def. 1)
 *       evaluated in exact arithmetic through its two thresholds:
 *         q = +1  iff  w' >= (0.5 - z) d ;   q = -1  iff  w' < (-0.5 - z) d ;   else 0
 *       (z integer, d an fp16 value: both products are exact in fp64).
 */
static uint32_t ref_quantize_block(const float *w, uint8_t *codes_out, uint32_t *flags)
{
    double a[ITQ3S_REF_BLOCK], e2[ITQ3S_REF_BLOCK];
    int finite = 1;
    for (int j = 0; j < ITQ3S_REF_BLOCK; j++) {
        a[j] = (double)w[j];
        if (!isfinite(a[j])) finite = 0;
    }
    if (!finite) {
        if (flags) *flags |= REF_FLAG_NONFINITE;
        memset(codes_out, 1, ITQ3S_REF_BLOCK);
        return 0u;
    }
    itq3s_ref_fwht256(a);
    for (int j = 0; j < ITQ3S_REF_BLOCK; j++) a[j] = a[j] * 0.0625;
    double mu = ref_pairwise_sum256(a) / 256.0;
    for (int j = 0; j < ITQ3S_REF_BLOCK; j++) {
        double dev = a[j] - mu;
        e2[j] = dev * dev;
    }
    double sigma = sqrt(ref_pairwise_sum256(e2) / 256.0);
    double d64 = ITQ3S_REF_T_STAR * sigma;
    if (d64 > 65504.0) {
        d64 = 65504.0;
        if (flags) *flags |= REF_FLAG_SCALE_SAT;
    }
    uint16_t dbits = ref_f32_to_f16((float)d64);
    double d = ref_f16_to_f64(dbits);
    if (!(d > 0.0)) { /* constant transform-domain block, or scale below the fp16 range */
        memset(codes_out, 1, ITQ3S_REF_BLOCK);
        return 0u;
    }
    double r = floor(mu / d + 0.5);
    double z = 0.0 - r;                                     /* +0 when r == 0 */
    if (z > 2048.0) { z = 2048.0; if (flags) *flags |= REF_FLAG_Z_CLAMP; }
    if (z < -2048.0) { z = -2048.0; if (flags) *flags |= REF_FLAG_Z_CLAMP; }
    double t_hi = (0.5 - z) * d, t_lo = (-0.5 - z) * d;
    for (int j = 0; j < ITQ3S_REF_BLOCK; j++) codes_out[j] = (uint8_t)(a[j] >= t_hi ? 2 : (a[j] < t_lo ? 0 : 1));
    uint16_t zbits = ref_f32_to_f16((float)z);              /* exact: |z| <= 2048 integer */
    return (uint32_t)dbits | ((uint32_t)zbits << 16);
}

/* W: N x K fp32, row stride ldw (elements).  codes/scales: sized by the _bytes helpers. */
int itq3s_ref_quantize(const float *W, int64_t N, int64_t K, int64_t ldw, uint32_t *codes, uint32_t *scales, uint32_t *flags)
{
    if (!W || !codes || !scales) return -1;
    if (N <= 0 || K <= 0 || (K % 256) != 0 || ldw < K) return -2;
    int64_t KB = K / 256, NT = (N + 15) / 16;
    uint8_t c[ITQ3S_REF_BLOCK];
    for (int64_t n = 0; n < NT * 16; n++)
        for (int64_t b = 0; b < KB; b++) {
            uint32_t word = 0;
            if (n < N) word = ref_quantize_block(W + n * ldw + b * 256, c, flags);
            else memset(c, 1, sizeof c);
            uint32_t *tile = codes + ref_tile_index(n, b, KB) * ITQ3S_REF_TILE_WORDS;
            for (int e = 0; e < ITQ3S_REF_BLOCK; e++) ref_put_code(tile, (int)(n & 15), e, c[e]);
            scales[ref_tile_index(n, b, KB) * 16 + (n & 15)] = word;
        }
    return 0;
}

/* ------------------------------------------------------------------ block-size ablation (Sec. 6, "Ablation: FWHT Block Size") */

/* The paper repeats the method with transform lengths n = 32 .. 512 (its table reports perplexity
 * and kernel overhead per n).  What can be computed without a model is the round trip itself:
 * per block of n consecutive channels  w' = H_n w,  d = T* sigma(w') -> fp16,  z,  codes (Alg. 1,
 * Def. 1 exactly as for n = 256), then  w_hat = H_n( d (q - z) )  (Alg. 2, Prop. 1).
 * H_n is the normalised Hadamard matrix H_u / sqrt(n); 1/sqrt(n) is irrational for n = 32, 128, 512,
 * so the factor is a fixed fp64 constant (the correctly rounded value) applied with one
 * multiplication, after the butterflies: w' = (H_u w) * c_n and w_hat = (d * (H_u (q - z))) * c_n.
 * For n = 256 every step coincides with the functions above. */
static double ref_inv_sqrt_n(int n)
{
    switch (n) {
    case 32: return 0.17677669529663687;
    case 64: return 0.125;
    case 128: return 0.08838834764831843;
    case 256: return 0.0625;
    case 512: return 0.044194173824159216;
    }
    return 0.0;
}

static void ref_fwht_n(double *a, int n)
{
    for (int step = 1; step < n; step <<= 1)
        for (int i = 0; i < n; i++)
            if ((i & step) == 0) {
                double u = a[i], v = a[i + step];
                a[i] = u + v;
                a[i + step] = u - v;
            }
}

static double ref_pairwise_sum_n(const double *v, int n)
{
    double t[512];
    memcpy(t, v, (size_t)n * sizeof(double));
    for (int step = 1; step < n; step <<= 1)
        for (int i = 0; i < n; i += 2 * step) t[i] = t[i] + t[i + step];
    return t[0];
}

/* W: N x K fp32 (row stride ldw), K a multiple of n, n in {32, 64, 128, 256, 512}.
 * codes_out (N*K bytes, may be NULL): code c = q+1 of every weight, row-major.
 * scales_out (N*(K/n) words, may be NULL): fp16 d | fp16 z << 16 per block, row-major.
 * what_out (N*K doubles, may be NULL): reconstructed weights, row-major.
 * Degenerate and non-finite blocks are handled as in the 256-point quantizer. */
int itq3s_ref_roundtrip_n(const float *W, int64_t N, int64_t K, int64_t ldw, int n, uint8_t *codes_out, uint32_t *scales_out,
                          double *what_out, uint32_t *flags)
{
    double cn = ref_inv_sqrt_n(n);
    if (!W) return -1;
    if (cn == 0.0 || N <= 0 || K <= 0 || (K % n) != 0 || ldw < K) return -2;
    int64_t KBn = K / n;
    double a[512], e2[512], m[512];
    uint8_t c[512];
    for (int64_t r = 0; r < N; r++)
        for (int64_t b = 0; b < KBn; b++) {
            const float *w = W + r * ldw + b * n;
            int finite = 1;
            uint32_t word = 0;
            for (int j = 0; j < n; j++) {
                a[j] = (double)w[j];
                if (!isfinite(a[j])) finite = 0;
                c[j] = 1;
            }
            double d = 0.0, z = 0.0;
            if (!finite) {
                if (flags) *flags |= REF_FLAG_NONFINITE;
            } else {
                ref_fwht_n(a, n);
                for (int j = 0; j < n; j++) a[j] = a[j] * cn;
                double mu = ref_pairwise_sum_n(a, n) / (double)n;
                for (int j = 0; j < n; j++) {
                    double dev = a[j] - mu;
                    e2[j] = dev * dev;
                }
                double sigma = sqrt(ref_pairwise_sum_n(e2, n) / (double)n);
                double d64 = ITQ3S_REF_T_STAR * sigma;
                if (d64 > 65504.0) {
                    d64 = 65504.0;
                    if (flags) *flags |= REF_FLAG_SCALE_SAT;
                }
                uint16_t dbits = ref_f32_to_f16((float)d64);
                d = ref_f16_to_f64(dbits);
                if (d > 0.0) {
                    double rr = floor(mu / d + 0.5);
                    z = 0.0 - rr;
                    if (z > 2048.0) { z = 2048.0; if (flags) *flags |= REF_FLAG_Z_CLAMP; }
                    if (z < -2048.0) { z = -2048.0; if (flags) *flags |= REF_FLAG_Z_CLAMP; }
                    double t_hi = (0.5 - z) * d, t_lo = (-0.5 - z) * d;
                    for (int j = 0; j < n; j++) c[j] = (uint8_t)(a[j] >= t_hi ? 2 : (a[j] < t_lo ? 0 : 1));
                    word = (uint32_t)dbits | ((uint32_t)ref_f32_to_f16((float)z) << 16);
                } else {
                    d = 0.0;
                }
            }
            if (codes_out) memcpy(codes_out + r * K + b * n, c, (size_t)n);
            if (scales_out) scales_out[r * KBn + b] = word;
            if (what_out) {
                for (int j = 0; j < n; j++) m[j] = (double)((int)c[j] - 1) - z;
                if (!(d > 0.0)) for (int j = 0; j < n; j++) m[j] = 0.0;
                ref_fwht_n(m, n);
                for (int j = 0; j < n; j++) what_out[r * K + b * n + j] = (d * m[j]) * cn;
            }
        }
    return 0;
}

/* ------------------------------------------------------------------ dequantize (Alg. 2, Prop. 1) */

/* w_hat = H ( d_k (q - z_k) ): unpack, subtract the code zero-point 1 and z_k, run the same
 * butterfly network, scale by d_k / 16.  q - z is a small integer, so the butterflies are exact
 * and the only rounding is none at all in fp64 (11-bit d times a < 2^20 integer times 2^-4). */
static void ref_dequantize_block(const uint32_t *tile, int r, uint32_t scale_word, double *out, uint32_t *flags)
{
    double d = ref_f16_to_f64((uint16_t)(scale_word & 0xffffu));
    double z = ref_f16_to_f64((uint16_t)(scale_word >> 16));
    double v[ITQ3S_REF_BLOCK];
    for (int e = 0; e < ITQ3S_REF_BLOCK; e++) {
        uint32_t c = ref_get_code(tile, r, e);
        if (c > 2u && flags) *flags |= REF_FLAG_BAD_CODE;
        v[e] = ((double)c - 1.0) - z;
    }
    itq3s_ref_fwht256(v);
    for (int e = 0; e < ITQ3S_REF_BLOCK; e++) out[e] = d * v[e] * 0.0625;
}

int itq3s_ref_dequantize(const uint32_t *codes, const uint32_t *scales, int64_t N, int64_t K, double *W_out, int64_t ldo, uint32_t *flags)
{
    if (!codes || !scales || !W_out) return -1;
    if (N <= 0 || K <= 0 || (K % 256) != 0 || ldo < K) return -2;
    int64_t KB = K / 256;
    for (int64_t n = 0; n < N; n++)
        for (int64_t b = 0; b < KB; b++) {
            size_t t = ref_tile_index(n, b, KB);
            ref_dequantize_block(codes + t * ITQ3S_REF_TILE_WORDS, (int)(n & 15), scales[t * 16 + (n & 15)], W_out + n * ldo + b * 256, flags);
        }
    return 0;
}

/* ------------------------------------------------------------------ matmul (problem statement) */

/* Y[m][n] = sum_k X[m][k] * w_hat[n][k], k ascending, everything in fp64.
 * X: fp16 bit patterns, M x K, row stride ldx.  Y: M x N doubles, row stride ldy.
 * Rows n0 <= n < n1 only (n0 = 0, n1 = N for all): lets a caller sample or split rows. */
int itq3s_ref_matmul_rows(const uint32_t *codes, const uint32_t *scales, int64_t N, int64_t K, const uint16_t *X, int64_t M,
                          int64_t ldx, double *Y, int64_t ldy, int64_t n0, int64_t n1)
{
    if (!codes || !scales || !X || !Y) return -1;
    if (N <= 0 || K <= 0 || M <= 0 || (K % 256) != 0 || ldx < K || ldy < N || n0 < 0 || n1 > N || n0 > n1) return -2;
    int64_t KB = K / 256;
    double *wrow = (double *)malloc((size_t)K * sizeof(double));
    double *xrow = (double *)malloc((size_t)M * (size_t)K * sizeof(double));
    if (!wrow || !xrow) { free(wrow); free(xrow); return -3; }
    for (int64_t m = 0; m < M; m++)
        for (int64_t k = 0; k < K; k++) xrow[m * K + k] = ref_f16_to_f64(X[m * ldx + k]);
    for (int64_t n = n0; n < n1; n++) {
        for (int64_t b = 0; b < KB; b++) {
            size_t t = ref_tile_index(n, b, KB);
            ref_dequantize_block(codes + t * ITQ3S_REF_TILE_WORDS, (int)(n & 15), scales[t * 16 + (n & 15)], wrow + b * 256, NULL);
        }
        for (int64_t m = 0; m < M; m++) {
            double acc = 0.0;
            const double *x = xrow + m * K;
            for (int64_t k = 0; k < K; k++) acc += x[k] * wrow[k];
            Y[m * ldy + n] = acc;
        }
    }
    free(wrow);
    free(xrow);
    return 0;
}

int itq3s_ref_matmul(const uint32_t *codes, const uint32_t *scales, int64_t N, int64_t K, const uint16_t *X, int64_t M, int64_t ldx,
                     double *Y, int64_t ldy)
{
    return itq3s_ref_matmul_rows(codes, scales, N, K, X, M, ldx, Y, ldy, 0, N);
}

/* ------------------------------------------------------------------ sub-block-scale variant (Sec. 4.1, "Block Structure") */

/* The paper lists, as an option "for higher fidelity", 8 fp16 sub-block scales for 8 sub-blocks of
 * 32 elements on top of d_k and z_k: 96 + 2 + 2 + 16 = 116 bytes per block, 3.625 bit/weight.  It
 * gives no formula for them.  Reading taken here (PARITY UNPINNED beyond the byte budget, the
 * reduction to the base format for sub-scales 1, and the dense definition in the tests):
 *   - the sub-blocks are 32 consecutive coefficients of the ROTATED block w' = H w (the domain the
 *     codes live in), sub-block j = coefficients 32j .. 32j+31;
 *   - d_k and z_k are exactly those of the base format (Alg. 1), so the first 100 bytes keep their
 *     meaning; the zero-point stays in units of d_k;
 *   - s_j is the step of sub-block j relative to d_k:  s_j = T* sigma_j / d_k  with sigma_j the
 *     deviation of the sub-block's coefficients about the BLOCK mean (population, over 32), i.e. the
 *     Sec. 3.3 rule "scale = T* x empirical standard deviation" applied per sub-block; rounded to fp16
 *     through fp32 like d_k, and the codes are decided against the rounded value;
 *   - code:  q = clamp(floor((w'/d_k + z_k) / s_j + 0.5), -1, 1)  -- Def. 1 with the digit step s_j --
 *     through the exact thresholds  w' >= (0.5 s_j - z) d  and  w' < (-0.5 s_j - z) d ; a sub-block
 *     with s_j = 0 stores digit 0 everywhere;
 *   - reconstruction (Prop. 1 with the digit scaled):  w_hat = H( d_k ( s_j q - z_k ) ).
 * Sub-scale storage: one uint32 per (tile, lane) at index tile*64 + lane, lane = 16*g + r for tile
 * row r and quarter g of the block: bits 0..15 = fp16 s_(2g), bits 16..31 = fp16 s_(2g+1)
 * (256 bytes per tile = 16 bytes per block). */

size_t itq3s_ref_subscales_bytes(int64_t N, int64_t K) { return (size_t)((N + 15) / 16) * (size_t)(K / 256) * 256u; }

static double ref_pairwise_sum32(const double *v)
{
    double t[32];
    memcpy(t, v, sizeof t);
    for (int step = 1; step < 32; step <<= 1)
        for (int i = 0; i < 32; i += 2 * step) t[i] = t[i] + t[i + step];
    return t[0];
}

/* One block: codes (256 bytes), 8 sub-scale bit patterns; returns the scale word of the base format. */
static uint32_t ref_quantize_block_sub(const float *w, uint8_t *codes_out, uint16_t *sub_out, uint32_t *flags)
{
    double a[ITQ3S_REF_BLOCK], e2[ITQ3S_REF_BLOCK];
    int finite = 1;
    memset(codes_out, 1, ITQ3S_REF_BLOCK);
    for (int j = 0; j < 8; j++) sub_out[j] = 0;
    for (int j = 0; j < ITQ3S_REF_BLOCK; j++) {
        a[j] = (double)w[j];
        if (!isfinite(a[j])) finite = 0;
    }
    if (!finite) {
        if (flags) *flags |= REF_FLAG_NONFINITE;
        return 0u;
    }
    itq3s_ref_fwht256(a);
    for (int j = 0; j < ITQ3S_REF_BLOCK; j++) a[j] = a[j] * 0.0625;
    double mu = ref_pairwise_sum256(a) / 256.0;
    for (int j = 0; j < ITQ3S_REF_BLOCK; j++) {
        double dev = a[j] - mu;
        e2[j] = dev * dev;
    }
    double sigma = sqrt(ref_pairwise_sum256(e2) / 256.0);
    double d64 = ITQ3S_REF_T_STAR * sigma;
    if (d64 > 65504.0) {
        d64 = 65504.0;
        if (flags) *flags |= REF_FLAG_SCALE_SAT;
    }
    uint16_t dbits = ref_f32_to_f16((float)d64);
    double d = ref_f16_to_f64(dbits);
    if (!(d > 0.0)) return 0u;
    double r = floor(mu / d + 0.5);
    double z = 0.0 - r;
    if (z > 2048.0) { z = 2048.0; if (flags) *flags |= REF_FLAG_Z_CLAMP; }
    if (z < -2048.0) { z = -2048.0; if (flags) *flags |= REF_FLAG_Z_CLAMP; }
    for (int j = 0; j < 8; j++) {
        double sigma_j = sqrt(ref_pairwise_sum32(e2 + 32 * j) / 32.0);
        double s64 = ITQ3S_REF_T_STAR * sigma_j / d;
        if (s64 > 65504.0) {
            s64 = 65504.0;
            if (flags) *flags |= REF_FLAG_SCALE_SAT;
        }
        sub_out[j] = ref_f32_to_f16((float)s64);
        double s = ref_f16_to_f64(sub_out[j]);
        if (!(s > 0.0)) continue; /* digit 0 everywhere */
        double t_hi = (0.5 * s - z) * d, t_lo = (-0.5 * s - z) * d;
        for (int i = 32 * j; i < 32 * j + 32; i++) codes_out[i] = (uint8_t)(a[i] >= t_hi ? 2 : (a[i] < t_lo ? 0 : 1));
    }
    uint16_t zbits = ref_f32_to_f16((float)z);
    return (uint32_t)dbits | ((uint32_t)zbits << 16);
}

int itq3s_ref_quantize_sub(const float *W, int64_t N, int64_t K, int64_t ldw, uint32_t *codes, uint32_t *scales, uint32_t *subs,
                           uint32_t *flags)
{
    if (!W || !codes || !scales || !subs) return -1;
    if (N <= 0 || K <= 0 || (K % 256) != 0 || ldw < K) return -2;
    int64_t KB = K / 256, NT = (N + 15) / 16;
    uint8_t c[ITQ3S_REF_BLOCK];
    uint16_t sb[8];
    for (int64_t n = 0; n < NT * 16; n++)
        for (int64_t b = 0; b < KB; b++) {
            uint32_t word = 0;
            if (n < N) word = ref_quantize_block_sub(W + n * ldw + b * 256, c, sb, flags);
            else {
                memset(c, 1, sizeof c);
                memset(sb, 0, sizeof sb);
            }
            size_t t = ref_tile_index(n, b, KB);
            uint32_t *tile = codes + t * ITQ3S_REF_TILE_WORDS;
            for (int e = 0; e < ITQ3S_REF_BLOCK; e++) ref_put_code(tile, (int)(n & 15), e, c[e]);
            scales[t * 16 + (n & 15)] = word;
            for (int g = 0; g < 4; g++) subs[t * 64 + 16 * g + (n & 15)] = (uint32_t)sb[2 * g] | ((uint32_t)sb[2 * g + 1] << 16);
        }
    return 0;
}

static void ref_dequantize_block_sub(const uint32_t *tile, const uint32_t *subs_tile, int r, uint32_t scale_word, double *out, uint32_t *flags)
{
    double d = ref_f16_to_f64((uint16_t)(scale_word & 0xffffu));
    double z = ref_f16_to_f64((uint16_t)(scale_word >> 16));
    double v[ITQ3S_REF_BLOCK];
    for (int e = 0; e < ITQ3S_REF_BLOCK; e++) {
        uint32_t c = ref_get_code(tile, r, e);
        if (c > 2u && flags) *flags |= REF_FLAG_BAD_CODE;
        int j = e >> 5; /* sub-block */
        uint32_t sw = subs_tile[16 * (j >> 1) + r];
        double s = ref_f16_to_f64((uint16_t)((j & 1) ? (sw >> 16) : (sw & 0xffffu)));
        v[e] = s * ((double)c - 1.0) - z;
    }
    itq3s_ref_fwht256(v);
    for (int e = 0; e < ITQ3S_REF_BLOCK; e++) out[e] = d * v[e] * 0.0625;
}

int itq3s_ref_dequantize_sub(const uint32_t *codes, const uint32_t *scales, const uint32_t *subs, int64_t N, int64_t K, double *W_out,
                             int64_t ldo, uint32_t *flags)
{
    if (!codes || !scales || !subs || !W_out) return -1;
    if (N <= 0 || K <= 0 || (K % 256) != 0 || ldo < K) return -2;
    int64_t KB = K / 256;
    for (int64_t n = 0; n < N; n++)
        for (int64_t b = 0; b < KB; b++) {
            size_t t = ref_tile_index(n, b, KB);
            ref_dequantize_block_sub(codes + t * ITQ3S_REF_TILE_WORDS, subs + t * 64, (int)(n & 15), scales[t * 16 + (n & 15)],
                                     W_out + n * ldo + b * 256, flags);
        }
    return 0;
}

/* Y = X W_hat^T for the sub-block variant, rows n0 <= n < n1, as itq3s_ref_matmul_rows. */
int itq3s_ref_matmul_sub_rows(const uint32_t *codes, const uint32_t *scales, const uint32_t *subs, int64_t N, int64_t K, const uint16_t *X,
                              int64_t M, int64_t ldx, double *Y, int64_t ldy, int64_t n0, int64_t n1)
{
    if (!codes || !scales || !subs || !X || !Y) return -1;
    if (N <= 0 || K <= 0 || M <= 0 || (K % 256) != 0 || ldx < K || ldy < N || n0 < 0 || n1 > N || n0 > n1) return -2;
    int64_t KB = K / 256;
    double *wrow = (double *)malloc((size_t)K * sizeof(double));
    double *xrow = (double *)malloc((size_t)M * (size_t)K * sizeof(double));
    if (!wrow || !xrow) { free(wrow); free(xrow); return -3; }
    for (int64_t m = 0; m < M; m++)
        for (int64_t k = 0; k < K; k++) xrow[m * K + k] = ref_f16_to_f64(X[m * ldx + k]);
    for (int64_t n = n0; n < n1; n++) {
        for (int64_t b = 0; b < KB; b++) {
            size_t t = ref_tile_index(n, b, KB);
            ref_dequantize_block_sub(codes + t * ITQ3S_REF_TILE_WORDS, subs + t * 64, (int)(n & 15), scales[t * 16 + (n & 15)], wrow + b * 256, NULL);
        }
        for (int64_t m = 0; m < M; m++) {
            double acc = 0.0;
            const double *x = xrow + m * K;
            for (int64_t k = 0; k < K; k++) acc += x[k] * wrow[k];
            Y[m * ldy + n] = acc;
        }
    }
    free(wrow);
    free(xrow);
    return 0;
}

uint32_t itq3s_ref_quantize_block_sub(const float *w, uint8_t *codes_out, uint16_t *sub_out, uint32_t *flags)
{
    return ref_quantize_block_sub(w, codes_out, sub_out, flags);
}

/* ------------------------------------------------------------------ small exports for the tests */

/* The forward normalised transform of one block, as the quantizer sees it (w' = H w). */
void itq3s_ref_forward_block(const float *w, double *wt)
{
    for (int j = 0; j < ITQ3S_REF_BLOCK; j++) wt[j] = (double)w[j];
    itq3s_ref_fwht256(wt);
    for (int j = 0; j < ITQ3S_REF_BLOCK; j++) wt[j] = wt[j] * 0.0625;
}

/* Quantize one block without packing: codes (256 bytes) and the scale word. */
uint32_t itq3s_ref_quantize_block(const float *w, uint8_t *codes_out, uint32_t *flags) { return ref_quantize_block(w, codes_out, flags); }

uint16_t itq3s_ref_f32_to_f16(float f) { return ref_f32_to_f16(f); }
double itq3s_ref_f16_to_f64(uint16_t h) { return ref_f16_to_f64(h); }
double itq3s_ref_t_star(void) { return ITQ3S_REF_T_STAR; }
