/*
 * mxfp4_ref.c -- CPU oracle for the FP8 <-> software-MXFP4 conversions.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, sequential statement of what
 * the conversions compute, written so that it can be checked against the paper by eye.
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may call it; the
 * GPU library never does, and the two share no source, tables or helpers.
 *
 * Formats (paper section 3.1 and 3.3):
 *   E4M3  : OCP float8_e4m3fn. bias 7, subnormals m/8 * 2^-6, max 448 (0x7E), NaN 0x7F/0xFF.
 *   E2M1  : 1 sign, 2 exponent (bias 1), 1 mantissa bit: magnitudes 0 .5 1 1.5 2 3 4 6.
 *   UE8M0 : byte b means 2^(b-127), b in [0,254]; 255 = NaN.
 *   FP8 activations carry one FP32 scale per 1x128 tile; MXFP4 one UE8M0 byte per 32.
 *
 * All floating-point work is done in double, where every quantity below is exact:
 * an E4M3 value has 4 significant bits, an FP32 scale 24, and everything after the
 * single FP32 rounding of their product is a comparison or a power-of-two scaling.
 *
 * Every function takes host pointers.  Return value: 0, or -1 for an argument error.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#define FP4_MAX 6.0 /* section 3.1: largest E2M1 magnitude */

/* ---------------------------------------------------------------- number formats */

/* Value of a 7-bit E4M3 magnitude code (sign stripped, code != 0x7F). */
static double e4m3_magnitude(unsigned code7)
{
    unsigned e = code7 >> 3, m = code7 & 7u;
    if (e == 0)
        return ldexp((double)m, -9); /* subnormal: (m/8) * 2^-6 */
    return ldexp(1.0 + (double)m / 8.0, (int)e - 7);
}

/* Value of a 3-bit E2M1 magnitude code. */
static double e2m1_magnitude(unsigned code3)
{
    unsigned e = code3 >> 1, m = code3 & 1u;
    if (e == 0)
        return 0.5 * (double)m; /* subnormal: no implicit bit */
    return ldexp(1.0 + 0.5 * (double)m, (int)e - 1);
}

/* Round-to-nearest, ties-to-even (section 3.1) of y >= 0 onto the E2M1 grid.
 * "Even" is the code whose mantissa bit is 0.  Anything above 6, and +inf, saturates. */
static unsigned e2m1_round_nearest_even(double y)
{
    if (!(y <= FP4_MAX))
        return 7u;
    unsigned best = 0;
    double best_err = y; /* distance to magnitude 0 */
    for (unsigned c = 1; c < 8; ++c) {
        double err = fabs(y - e2m1_magnitude(c));
        if (err < best_err || (err == best_err && (c & 1u) == 0u)) {
            best = c;
            best_err = err;
        }
    }
    return best;
}

/* Round-to-nearest, ties-to-even of 0 <= r <= 448 onto the E4M3 grid (subnormals
 * included: gradual underflow).  grid[c] holds e4m3_magnitude(c) for c = 0..0x7E. */
static unsigned e4m3_round_nearest_even(double r, const double *grid)
{
    unsigned best = 0;
    double best_err = r;
    for (unsigned c = 1; c <= 0x7Eu; ++c) {
        double err = fabs(r - grid[c]);
        if (err < best_err || (err == best_err && (c & 1u) == 0u)) {
            best = c;
            best_err = err;
        }
    }
    return best;
}

/* The MXFP4 block scale of section 3.1: SF = 2^ceil(log2(gmax / 6)), i.e. the smallest
 * power of two 2^k with gmax <= 6 * 2^k, stored as the byte k+127 clamped to [0,254].
 * gmax must be finite and > 0.  frexp gives gmax = f * 2^e with 0.5 <= f < 1, so
 * gmax <= 6*2^k  <=>  f * 2^e <= 0.75 * 2^(k+3)  <=>  k >= e-3 (f <= .75) or e-2. */
static int ue8m0_byte_for_block_max(double gmax)
{
    int e;
    double f = frexp(gmax, &e);
    int k = (f <= 0.75) ? e - 3 : e - 2;
    int b = k + 127;
    if (b < 0)
        b = 0;
    if (b > 254)
        b = 254;
    return b;
}

/* Quantize 32 exact real values v[0..31] (sign and magnitude, doubles; may be +-inf)
 * to one MXFP4 block: the scale rule and rounding of section 3.1.
 * has_nan != 0 marks a block that contains a NaN.  code[i] receives the 4-bit code
 * (sign << 3 | magnitude).  Returns the scale byte. */
static unsigned quantize_block32(const double *v, int has_nan, unsigned char *code)
{
    if (has_nan) { /* a NaN poisons the block: scale byte NaN, codes zero */
        for (int i = 0; i < 32; ++i)
            code[i] = 0;
        return 0xFFu;
    }
    double gmax = 0.0;
    for (int i = 0; i < 32; ++i)
        if (fabs(v[i]) > gmax)
            gmax = fabs(v[i]);

    int b;
    if (gmax == 0.0)
        b = 0; /* a zero block has a zero scale byte */
    else if (isinf(gmax))
        b = 254;
    else
        b = ue8m0_byte_for_block_max(gmax);

    for (int i = 0; i < 32; ++i) {
        double y = ldexp(fabs(v[i]), -(b - 127)); /* exact: power-of-two scaling */
        unsigned mag = e2m1_round_nearest_even(y);
        unsigned sign = signbit(v[i]) ? 1u : 0u; /* the sign is always copied, -0 too */
        code[i] = (unsigned char)((sign << 3) | mag);
    }
    return (unsigned)b;
}

/* ---------------------------------------------------------------- FP8 -> MXFP4 */

/* E4M3 [M_src,K] with FP32 scales [M_src,K/128]  ->  packed E2M1 [M_out, K/2] (row
 * stride ld_q bytes) and UE8M0 [M_out, K/32] (row stride ld_sf bytes).
 * gather_idx == NULL: row i of the output comes from row i of the input (M_out == M_src);
 * otherwise from row gather_idx[i].
 * The value of an element is its blockwise-FP8 dequantized FP32 value fl32(e4m3 * s):
 * one rounding to FP32, subnormals kept; section 3.1's quantizer is applied to it.
 * The product follows IEEE-754 also for scales outside the format's range: a NaN scale, or an
 * infinite scale times a zero element, gives a NaN element (which poisons its block like a NaN code).
 * Packing: byte j of a row holds element 2j in bits 3..0 and element 2j+1 in bits 7..4. */
int mxfp4_ref_quant_from_fp8(const uint8_t *x, const float *x_scale, int64_t M_src, int64_t K,
                             const int32_t *gather_idx, int64_t M_out, uint8_t *q, int64_t ld_q,
                             uint8_t *sf, int64_t ld_sf)
{
    if (M_src < 0 || M_out < 0 || K < 0 || K % 128 != 0)
        return -1;
    if (M_out == 0 || K == 0)
        return 0;
    if (!x || !x_scale || !q || !sf || ld_q < K / 2 || ld_sf < K / 32)
        return -1;
    if (!gather_idx && M_out != M_src)
        return -1;

    for (int64_t i = 0; i < M_out; ++i) {
        int64_t r = gather_idx ? (int64_t)gather_idx[i] : i;
        if (r < 0 || r >= M_src)
            return -1;
        for (int64_t j = 0; j < K / 32; ++j) {
            double s = (double)x_scale[r * (K / 128) + j / 4];
            double v[32];
            int has_nan = 0;
            for (int e = 0; e < 32; ++e) {
                unsigned c = x[r * K + j * 32 + e];
                if ((c & 0x7Fu) == 0x7Fu) {
                    has_nan = 1;
                    v[e] = 0.0;
                    continue;
                }
                double a = e4m3_magnitude(c & 0x7Fu);
                float p = (float)(a * s); /* the product is exact in double; one rounding to FP32 */
                if (isnan(p)) { /* NaN scale, or 0 * inf */
                    has_nan = 1;
                    v[e] = 0.0;
                    continue;
                }
                v[e] = (c & 0x80u) ? -(double)p : (double)p;
            }
            unsigned char code[32];
            unsigned b = quantize_block32(v, has_nan, code);
            sf[i * ld_sf + j] = (uint8_t)b;
            for (int e = 0; e < 16; ++e)
                q[i * ld_q + j * 16 + e] = (uint8_t)(code[2 * e] | (code[2 * e + 1] << 4));
        }
    }
    return 0;
}

/* ---------------------------------------------------------------- BF16 -> MXFP4 */

/* Value of a BF16 bit pattern (the upper half of an FP32); NaN and +-inf as such. */
static double bf16_value(unsigned h)
{
    unsigned sign = h >> 15, e = (h >> 7) & 0xFFu, m = h & 0x7Fu;
    double a;
    if (e == 0xFFu)
        a = m ? NAN : INFINITY;
    else if (e == 0)
        a = ldexp((double)m, -133); /* subnormal: (m/128) * 2^-126 */
    else
        a = ldexp(1.0 + (double)m / 128.0, (int)e - 127);
    return sign ? -a : a;
}

/* The row-wise quantizer as the paper states it (section 3.1, BF16 input): BF16 [M,K] ->
 * packed E2M1 [M,K/2] (row stride ld_q) + UE8M0 [M,K/32] (row stride ld_sf).  The element
 * values are the BF16 values themselves.  K % 128 == 0 like everywhere in this library. */
int mxfp4_ref_quant_from_bf16(const uint16_t *x, int64_t M, int64_t K, uint8_t *q, int64_t ld_q, uint8_t *sf,
                              int64_t ld_sf)
{
    if (M < 0 || K < 0 || K % 128 != 0)
        return -1;
    if (M == 0 || K == 0)
        return 0;
    if (!x || !q || !sf || ld_q < K / 2 || ld_sf < K / 32)
        return -1;
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < K / 32; ++j) {
            double v[32];
            int has_nan = 0;
            for (int e = 0; e < 32; ++e) {
                v[e] = bf16_value(x[i * K + j * 32 + e]);
                if (isnan(v[e])) {
                    has_nan = 1;
                    v[e] = 0.0;
                }
            }
            unsigned char code[32];
            unsigned b = quantize_block32(v, has_nan, code);
            sf[i * ld_sf + j] = (uint8_t)b;
            for (int e = 0; e < 16; ++e)
                q[i * ld_q + j * 16 + e] = (uint8_t)(code[2 * e] | (code[2 * e + 1] << 4));
        }
    }
    return 0;
}

/* The same quantizer with the routing turned around (section 3.2: quantization sits right before
 * the dispatch, so a token is quantized once and its packed row goes to each of its experts):
 * source row i is written to the output rows dst_idx[i*fanout + j], j < fanout; an entry outside
 * [0, M_out) is skipped; output rows that no entry names are left as they are.  Every output row
 * may be named at most once. */
int mxfp4_ref_quant_from_fp8_scatter(const uint8_t *x, const float *x_scale, int64_t M_src, int64_t K,
                                     const int32_t *dst_idx, int32_t fanout, int64_t M_out, uint8_t *q,
                                     int64_t ld_q, uint8_t *sf, int64_t ld_sf)
{
    if (M_src < 0 || M_out < 0 || K < 0 || K % 128 != 0 || fanout <= 0)
        return -1;
    if (M_src == 0 || M_out == 0 || K == 0)
        return 0;
    if (!x || !x_scale || !dst_idx || !q || !sf || ld_q < K / 2 || ld_sf < K / 32)
        return -1;
    for (int64_t i = 0; i < M_src; ++i) {
        for (int32_t j = 0; j < fanout; ++j) {
            int64_t d = dst_idx[i * fanout + j];
            if (d < 0 || d >= M_out)
                continue;
            int rc = mxfp4_ref_quant_from_fp8(x + i * K, x_scale + i * (K / 128), 1, K, NULL, 1, q + d * ld_q, ld_q,
                                              sf + d * ld_sf, ld_sf);
            if (rc)
                return rc;
        }
    }
    return 0;
}

/* ---------------------------------------------------------------- MXFP4 -> FP8 */

/* Packed E2M1 [M,K/2] + UE8M0 [M,K/32]  ->  E4M3 [M,K] + FP32 scale per 1x128 tile
 * [M,K/128]: the direct conversion with hierarchical scale alignment (section 3.3,
 * Algorithm 1).  Per tile with scale bytes b_0..b_3:
 *   tile scale   = 2^(max(b) - 6 - 127)          (Algorithm 1 step 1, delta = 6)
 *   element      = e2m1(code) * 2^(6 - (max(b) - b_i)) rounded to nearest-even E4M3,
 *                  which for normal codes and a non-negative E4M3 exponent is the
 *                  exponent re-bias E_fp4 - 1 + 7 minus the alignment shift, with the
 *                  mantissa bit moved to the E4M3 mantissa MSB (Algorithm 1 steps 2-8).
 * The E2M1 codes 0 and 1 (zero and the subnormal 0.5) take their true values, and an
 * exponent that would fall below 1 rounds into the E4M3 subnormals, then to zero.
 * A NaN scale byte (0xFF) makes the tile scale NaN and that block's 32 outputs 0x7F;
 * the other blocks of the tile align to the maximum of the non-NaN bytes. */
int mxfp4_ref_dequant_to_fp8(const uint8_t *q, int64_t ld_q, const uint8_t *sf, int64_t ld_sf,
                             int64_t M, int64_t K, uint8_t *x, float *x_scale)
{
    if (M < 0 || K < 0 || K % 128 != 0)
        return -1;
    if (M == 0 || K == 0)
        return 0;
    if (!q || !sf || !x || !x_scale || ld_q < K / 2 || ld_sf < K / 32)
        return -1;

    double grid[0x7F];
    for (unsigned c = 0; c <= 0x7Eu; ++c)
        grid[c] = e4m3_magnitude(c);

    for (int64_t i = 0; i < M; ++i) {
        for (int64_t t = 0; t < K / 128; ++t) {
            const uint8_t *b = sf + i * ld_sf + t * 4;
            int bmax = 0, any_nan = 0;
            for (int j = 0; j < 4; ++j) {
                if (b[j] == 0xFFu)
                    any_nan = 1;
                else if (b[j] > bmax)
                    bmax = b[j];
            }
            int b8 = bmax - 6;
            x_scale[i * (K / 128) + t] = any_nan ? (float)NAN : (float)ldexp(1.0, b8 - 127);

            for (int j = 0; j < 4; ++j) {
                for (int e = 0; e < 32; ++e) {
                    int64_t k = t * 128 + j * 32 + e;
                    unsigned byte = q[i * ld_q + k / 2];
                    unsigned nib = (k & 1) ? (byte >> 4) : (byte & 0xFu);
                    uint8_t out;
                    if (b[j] == 0xFFu) {
                        out = 0x7Fu;
                    } else {
                        int d = bmax - (int)b[j];
                        double r = ldexp(e2m1_magnitude(nib & 7u), 6 - d);
                        out = (uint8_t)(((nib >> 3) << 7) | e4m3_round_nearest_even(r, grid));
                    }
                    x[i * K + k] = out;
                }
            }
        }
    }
    return 0;
}

/* ---------------------------------------------------------------- row-blocked -> column-blocked */

/* Row-blocked MXFP4 (nibbles [M,K/2], 1x32 scales [M,K/32]) -> column-blocked MXFP4 of
 * the same matrix, stored transposed: nibbles [K,ceil(M/2)] (low nibble = even m) and 32x1
 * scales [K,ceil(M/32)].  Definition (section 3.4: de-quantization, transposition and
 * re-quantization in one pass): every element takes its exact real value
 * +-e2m1(code) * 2^(b_row - 127); each run of 32 consecutive m at fixed k is then
 * quantized with the scale rule and rounding of section 3.1.  A last run of fewer than 32 rows
 * (ragged splits only) is quantized over the rows it has; with an odd M the unused high nibble
 * of a k-row's last byte is 0.  A NaN row scale poisons every column block it touches. */
static void col_blocks_of_rows(const uint8_t *q_row, const uint8_t *sf_row, int64_t M, int64_t K,
                               uint8_t *q_col, uint8_t *sf_col)
{
    const int64_t B = (M + 31) / 32, P = (M + 1) / 2; /* blocks and bytes per output row */
    for (int64_t k = 0; k < K; ++k) {
        for (int64_t mb = 0; mb < B; ++mb) {
            const int n = (int)(M - mb * 32 < 32 ? M - mb * 32 : 32);
            double v[32];
            int has_nan = 0;
            for (int e = 0; e < 32; ++e) {
                v[e] = 0.0; /* rows that do not exist count as zeros and are not stored */
                if (e >= n)
                    continue;
                int64_t m = mb * 32 + e;
                unsigned byte = q_row[m * (K / 2) + k / 2];
                unsigned nib = (k & 1) ? (byte >> 4) : (byte & 0xFu);
                unsigned b = sf_row[m * (K / 32) + k / 32];
                if (b == 0xFFu) {
                    has_nan = 1;
                    continue;
                }
                double a = ldexp(e2m1_magnitude(nib & 7u), (int)b - 127);
                v[e] = (nib & 8u) ? -a : a;
            }
            unsigned char code[32];
            unsigned bc = quantize_block32(v, has_nan, code);
            sf_col[k * B + mb] = (uint8_t)bc;
            for (int e = 0; e < (n + 1) / 2; ++e) {
                unsigned hi = 2 * e + 1 < n ? code[2 * e + 1] : 0u;
                q_col[k * P + mb * 16 + e] = (uint8_t)(code[2 * e] | (hi << 4));
            }
        }
    }
}

/* The flat conversion: M % 32 == 0. */
int mxfp4_ref_row_to_col(const uint8_t *q_row, const uint8_t *sf_row, int64_t M, int64_t K,
                         uint8_t *q_col, uint8_t *sf_col)
{
    if (M < 0 || K < 0 || K % 128 != 0 || M % 32 != 0)
        return -1;
    if (M == 0 || K == 0)
        return 0;
    if (!q_row || !sf_row || !q_col || !sf_col)
        return -1;
    col_blocks_of_rows(q_row, sf_row, M, K, q_col, sf_col);
    return 0;
}

/* ---------------------------------------------------------------- row-blocked MXFP4 -> column-wise FP8 */

/* Row-blocked MXFP4 (nibbles [M,K/2], 1x32 scales [M,K/32]) -> the transposed matrix as FP8:
 * E4M3 [K,M] plus one FP32 scale per 128 consecutive m at fixed k, [K,ceil(M/128)] (the layout the
 * weight-gradient GEMM reads; section 3.4's fused de-quantization + transposition +
 * re-quantization, with the FP4 -> FP8 step of section 3.3 / Algorithm 1 taken along m).
 * For output row k and the rows m of group g (128 of them; fewer in a last, partial group of a
 * ragged split), with b_m = sf_row[m][k/32]:
 *   scale[k][g] = 2^(max_m(b_m) - 6 - 127)                       (Algorithm 1 step 1)
 *   x[k][m]     = e2m1(code[m][k]) * 2^(6 - (max(b) - b_m)) rounded to nearest-even E4M3
 * exactly as in mxfp4_ref_dequant_to_fp8, the aligned "blocks" now being the single elements
 * of the column.  A NaN scale byte makes the scale NaN and that row's element 0x7F; the other
 * rows align to the maximum of the non-NaN bytes. */
#define FP8_COL_ALIGN 0   /* Algorithm 1's scale alignment along m */
#define FP8_COL_REQUANT 1 /* re-quantization from the group's maximum, see below */

static void fp8_col_requant_group(const uint8_t *q_row, const uint8_t *sf_row, int64_t K, int64_t k, int64_t m0,
                                  int n, const double *grid, uint8_t *x_row, float *scale);

static void fp8_col_of_rows(const uint8_t *q_row, const uint8_t *sf_row, int64_t M, int64_t K,
                            uint8_t *x_col, float *x_col_scale, int rule)
{
    const int64_t G = (M + 127) / 128;
    double grid[0x7F];
    for (unsigned c = 0; c <= 0x7Eu; ++c)
        grid[c] = e4m3_magnitude(c);

    for (int64_t k = 0; k < K; ++k) {
        for (int64_t g = 0; g < G; ++g) {
            const int n = (int)(M - g * 128 < 128 ? M - g * 128 : 128); /* rows in this group */
            if (rule == FP8_COL_REQUANT) {
                fp8_col_requant_group(q_row, sf_row, K, k, g * 128, n, grid, x_col + k * M + g * 128,
                                      &x_col_scale[k * G + g]);
                continue;
            }
            int bmax = 0, any_nan = 0;
            for (int e = 0; e < n; ++e) {
                unsigned b = sf_row[(g * 128 + e) * (K / 32) + k / 32];
                if (b == 0xFFu)
                    any_nan = 1;
                else if ((int)b > bmax)
                    bmax = (int)b;
            }
            x_col_scale[k * G + g] = any_nan ? (float)NAN : (float)ldexp(1.0, bmax - 6 - 127);
            for (int e = 0; e < n; ++e) {
                int64_t m = g * 128 + e;
                unsigned b = sf_row[m * (K / 32) + k / 32];
                unsigned byte = q_row[m * (K / 2) + k / 2];
                unsigned nib = (k & 1) ? (byte >> 4) : (byte & 0xFu);
                uint8_t out;
                if (b == 0xFFu) {
                    out = 0x7Fu;
                } else {
                    double r = ldexp(e2m1_magnitude(nib & 7u), 6 - (bmax - (int)b));
                    out = (uint8_t)(((nib >> 3) << 7) | e4m3_round_nearest_even(r, grid));
                }
                x_col[k * M + m] = out;
            }
        }
    }
}

/* The other reading of the fused kernel (section 3.4: "de-quantization, transposition and
 * re-quantization", with the power-of-two scale 2^ceil(log2 x) of its bit-level arithmetic item):
 * the n elements of one output row k and one group take their exact values
 * v_m = +-e2m1(code) * 2^(b_m - 127); the group scale is the smallest power of two S with
 * max|v| / S <= 448 (the largest E4M3 magnitude), 1.0 for an all-zero group; every element is
 * v_m / S rounded to nearest-even E4M3 (gradual underflow; no saturation can occur).
 * A NaN scale byte makes the scale NaN and its row's element 0x7F; the maximum is taken over the
 * other rows. */
static void fp8_col_requant_group(const uint8_t *q_row, const uint8_t *sf_row, int64_t K, int64_t k, int64_t m0,
                                  int n, const double *grid, uint8_t *x_row, float *scale)
{
    double amax = 0.0;
    int any_nan = 0;
    for (int e = 0; e < n; ++e) {
        unsigned b = sf_row[(m0 + e) * (K / 32) + k / 32];
        unsigned byte = q_row[(m0 + e) * (K / 2) + k / 2];
        unsigned nib = (k & 1) ? (byte >> 4) : (byte & 0xFu);
        if (b == 0xFFu) {
            any_nan = 1;
            continue;
        }
        double a = ldexp(e2m1_magnitude(nib & 7u), (int)b - 127);
        if (a > amax)
            amax = a;
    }
    int j = 0; /* S = 2^j */
    if (amax > 0.0) {
        int ex;
        frexp(amax, &ex);
        j = ex - 12;                    /* 448 * 2^(ex-12) < 2^(ex-1) <= amax: too small, step up */
        while (amax > ldexp(448.0, j))  /* exact comparisons: both sides are doubles without rounding */
            ++j;
    }
    *scale = any_nan ? (float)NAN : (float)ldexp(1.0, j);
    for (int e = 0; e < n; ++e) {
        unsigned b = sf_row[(m0 + e) * (K / 32) + k / 32];
        unsigned byte = q_row[(m0 + e) * (K / 2) + k / 2];
        unsigned nib = (k & 1) ? (byte >> 4) : (byte & 0xFu);
        if (b == 0xFFu) {
            x_row[e] = 0x7Fu;
            continue;
        }
        double r = ldexp(e2m1_magnitude(nib & 7u), (int)b - 127 - j);
        x_row[e] = (uint8_t)(((nib >> 3) << 7) | e4m3_round_nearest_even(r, grid));
    }
}

/* The flat conversion: M % 128 == 0, scales [K, M/128]. */
int mxfp4_ref_row_to_fp8_col(const uint8_t *q_row, const uint8_t *sf_row, int64_t M, int64_t K,
                             uint8_t *x_col, float *x_col_scale)
{
    if (M < 0 || K < 0 || K % 128 != 0 || M % 128 != 0)
        return -1;
    if (M == 0 || K == 0)
        return 0;
    if (!q_row || !sf_row || !x_col || !x_col_scale)
        return -1;
    fp8_col_of_rows(q_row, sf_row, M, K, x_col, x_col_scale, FP8_COL_ALIGN);
    return 0;
}

int mxfp4_ref_row_to_fp8_col_requant(const uint8_t *q_row, const uint8_t *sf_row, int64_t M, int64_t K,
                                     uint8_t *x_col, float *x_col_scale)
{
    if (M < 0 || K < 0 || K % 128 != 0 || M % 128 != 0)
        return -1;
    if (M == 0 || K == 0)
        return 0;
    if (!q_row || !sf_row || !x_col || !x_col_scale)
        return -1;
    fp8_col_of_rows(q_row, sf_row, M, K, x_col, x_col_scale, FP8_COL_REQUANT);
    return 0;
}

/* ---------------------------------------------------------------- ragged (per-expert) variants */

/* expert_offsets[0..num_experts]: rows [off_e, off_{e+1}) belong to expert e (section 3.4,
 * ragged MoE tensors).  off_0 = 0, off_E = M_total, non-decreasing; any T_e >= 0.
 * Quantization is row-independent, so the grouped form is the flat form on M_total rows. */
static int offsets_ok(const int32_t *off, int32_t E, int64_t M_total)
{
    if (E <= 0 || !off || off[0] != 0 || (int64_t)off[E] != M_total)
        return 0;
    for (int32_t e = 0; e < E; ++e)
        if (off[e + 1] < off[e])
            return 0;
    return 1;
}

int mxfp4_ref_quant_from_fp8_grouped(const uint8_t *x, const float *x_scale,
                                     const int32_t *expert_offsets, int32_t num_experts,
                                     int64_t M_total, int64_t K, uint8_t *q, uint8_t *sf)
{
    if (!offsets_ok(expert_offsets, num_experts, M_total) || K < 0 || K % 128 != 0)
        return -1;
    for (int32_t e = 0; e < num_experts; ++e) {
        int64_t o = expert_offsets[e], T = expert_offsets[e + 1] - o;
        int rc = mxfp4_ref_quant_from_fp8(x ? x + o * K : x, x_scale ? x_scale + o * (K / 128) : x_scale, T,
                                          K, NULL, T, q ? q + o * (K / 2) : q, K / 2,
                                          sf ? sf + o * (K / 32) : sf, K / 32);
        if (rc)
            return rc;
    }
    return 0;
}

/* Ragged splits without padding (section 3.4): any T_e >= 0.  Expert e's output is its own dense
 * [K, ceil(T_e/2)] and [K, ceil(T_e/32)] matrices, stored back to back at byte offsets
 * K * sum_{j<e} ceil(T_j/2) and K * sum_{j<e} ceil(T_j/32) (= K*off_e/2 and K*off_e/32 when every
 * T_e is a multiple of 32). */
int mxfp4_ref_row_to_col_grouped(const uint8_t *q_row, const uint8_t *sf_row,
                                 const int32_t *expert_offsets, int32_t num_experts,
                                 int64_t M_total, int64_t K, uint8_t *q_col, uint8_t *sf_col)
{
    if (num_experts <= 0 || !expert_offsets || expert_offsets[0] != 0 ||
        (int64_t)expert_offsets[num_experts] != M_total || K < 0 || K % 128 != 0)
        return -1;
    for (int32_t e = 0; e < num_experts; ++e)
        if (expert_offsets[e + 1] < expert_offsets[e])
            return -1;
    if (M_total == 0 || K == 0)
        return 0;
    if (!q_row || !sf_row || !q_col || !sf_col)
        return -1;
    int64_t bytes_before = 0, blocks_before = 0;
    for (int32_t e = 0; e < num_experts; ++e) {
        int64_t o = expert_offsets[e], T = expert_offsets[e + 1] - o;
        if (T > 0)
            col_blocks_of_rows(q_row + o * (K / 2), sf_row + o * (K / 32), T, K, q_col + bytes_before * K,
                               sf_col + blocks_before * K);
        bytes_before += (T + 1) / 2;
        blocks_before += (T + 31) / 32;
    }
    return 0;
}

/* Ragged splits without padding (section 3.4): any T_e >= 0.  Expert e's FP8 output is its own
 * dense [K, T_e] matrix at element offset K*off_e, and its scales are its own dense
 * [K, ceil(T_e/128)] matrix at element offset K * sum_{j<e} ceil(T_j/128); a last group of fewer
 * than 128 rows takes its maximum over the rows it has.  With every T_e a multiple of 128 the
 * scale offset is K*off_e/128. */
static int fp8_col_grouped(const uint8_t *q_row, const uint8_t *sf_row, const int32_t *expert_offsets,
                           int32_t num_experts, int64_t M_total, int64_t K, uint8_t *x_col, float *x_col_scale,
                           int rule)
{
    if (num_experts <= 0 || !expert_offsets || expert_offsets[0] != 0 ||
        (int64_t)expert_offsets[num_experts] != M_total || K < 0 || K % 128 != 0)
        return -1;
    for (int32_t e = 0; e < num_experts; ++e)
        if (expert_offsets[e + 1] < expert_offsets[e])
            return -1;
    if (M_total == 0 || K == 0)
        return 0;
    if (!q_row || !sf_row || !x_col || !x_col_scale)
        return -1;
    int64_t groups_before = 0;
    for (int32_t e = 0; e < num_experts; ++e) {
        int64_t o = expert_offsets[e], T = expert_offsets[e + 1] - o;
        if (T > 0)
            fp8_col_of_rows(q_row + o * (K / 2), sf_row + o * (K / 32), T, K, x_col + o * K,
                            x_col_scale + groups_before * K, rule);
        groups_before += (T + 127) / 128;
    }
    return 0;
}

int mxfp4_ref_row_to_fp8_col_grouped(const uint8_t *q_row, const uint8_t *sf_row,
                                     const int32_t *expert_offsets, int32_t num_experts,
                                     int64_t M_total, int64_t K, uint8_t *x_col, float *x_col_scale)
{
    return fp8_col_grouped(q_row, sf_row, expert_offsets, num_experts, M_total, K, x_col, x_col_scale,
                           FP8_COL_ALIGN);
}

int mxfp4_ref_row_to_fp8_col_requant_grouped(const uint8_t *q_row, const uint8_t *sf_row,
                                             const int32_t *expert_offsets, int32_t num_experts,
                                             int64_t M_total, int64_t K, uint8_t *x_col, float *x_col_scale)
{
    return fp8_col_grouped(q_row, sf_row, expert_offsets, num_experts, M_total, K, x_col, x_col_scale,
                           FP8_COL_REQUANT);
}

/* ---------------------------------------------------------------- scalar entry points for the pins */

double mxfp4_ref_e4m3_value(unsigned byte)
{
    if ((byte & 0x7Fu) == 0x7Fu)
        return NAN;
    double a = e4m3_magnitude(byte & 0x7Fu);
    return (byte & 0x80u) ? -a : a;
}

double mxfp4_ref_e2m1_value(unsigned nibble)
{
    double a = e2m1_magnitude(nibble & 7u);
    return (nibble & 8u) ? -a : a;
}

unsigned mxfp4_ref_e2m1_round(double y) { return e2m1_round_nearest_even(y); }

unsigned mxfp4_ref_e4m3_round(double r)
{
    double grid[0x7F];
    for (unsigned c = 0; c <= 0x7Eu; ++c)
        grid[c] = e4m3_magnitude(c);
    return e4m3_round_nearest_even(r, grid);
}

int mxfp4_ref_scale_byte(double gmax) { return ue8m0_byte_for_block_max(gmax); }
