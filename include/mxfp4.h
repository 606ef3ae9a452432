/*
 * mxfp4.h -- C ABI of libmxfp4: direct conversions between DeepSeek-V3-style blockwise FP8
 * activations and software MXFP4 on AMD MI355X (gfx950).
 *
 * Formats
 *   FP8 side   : E4M3 bytes (OCP float8_e4m3fn: bias 7, max 448, NaN 0x7F/0xFF, no inf),
 *                dense row-major [M, K], plus one FP32 scale per 1x128 tile, [M, K/128].
 *                An element's value is fl32(e4m3 * scale).
 *   MXFP4 side : E2M1 codes (sign, 2 exponent bits bias 1, 1 mantissa bit; magnitudes
 *                0 .5 1 1.5 2 3 4 6) packed two per byte -- element 2j in bits 3..0 and
 *                element 2j+1 in bits 7..4 of byte j -- plus one UE8M0 byte per 32
 *                elements (byte b = 2^(b-127), b in [0,254]; 0xFF = NaN).
 *                "Row-blocked": blocks of 1x32 along K, nibbles [M, K/2], scales [M, K/32].
 *                "Column-blocked": blocks of 32x1 along M, stored transposed: nibbles
 *                [K, M/2] (even m in the low nibble), scales [K, M/32].
 *   Payloads   : FP8 = M*K + 4*M*K/128 bytes, MXFP4 = M*K/2 + M*K/32 bytes (paper sec. 3.2).
 *
 * Conventions (all entry points)
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library never
 *     allocates, frees, copies to the host or synchronises; a call enqueues its kernels on
 *     `hip_stream` (a hipStream_t passed as void*; NULL = the default stream) and returns.
 *   - Outputs must not alias inputs.  Buffers are row-major; K % 128 == 0.
 *   - Return value: MXFP4_OK, or a negative status; on an error nothing is launched.
 *     M == 0 (or K == 0) is MXFP4_OK and launches nothing.
 *   - Only host-visible arguments are validated.  The contents of device arrays
 *     (gather indices, expert offsets) are trusted; an out-of-range gather index yields a
 *     zero row rather than an out-of-bounds read.
 *   - NaN: an E4M3 NaN makes its MXFP4 block's scale byte 0xFF and its 16 packed bytes 0;
 *     a 0xFF scale byte makes the FP8 tile scale NaN and its block's 32 bytes 0x7F; in the
 *     row->column conversion it makes every column block it touches 0xFF / 0.
 *     Blockwise FP8 carries finite positive FP32 tile scales; what any other value does is stated at
 *     mxfp4_quant_from_fp8 (the IEEE-754 product decides).
 */
#ifndef MXFP4_H
#define MXFP4_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int mxfp4_status;

enum {
    MXFP4_OK = 0,
    MXFP4_ERR_NULL = -1,    /* a required pointer is NULL */
    MXFP4_ERR_SHAPE = -2,   /* negative size, K % 128 != 0, M % 32 != 0 (M % 128 != 0 for FP8
                               output) where column blocks are formed, a row stride smaller than the row, or a size beyond
                               what the 32-bit work indices of a kernel can address */
    MXFP4_ERR_ALIGN = -3,   /* pointer or row stride not aligned as stated per entry point */
    MXFP4_ERR_OFFSETS = -4, /* grouped: num_experts <= 0 or beyond MXFP4_MAX_EXPERTS */
    MXFP4_ERR_LAUNCH = -5   /* the HIP runtime reported an error at launch */
};

#define MXFP4_MAX_EXPERTS 1024

/* FP8 -> MXFP4 (paper sec. 3.1: per 1x32 block SF = 2^ceil(log2(max|v| / 6)) as UE8M0, then
 * round-to-nearest, ties-to-even onto E2M1 with gradual underflow and saturation; applied
 * directly to the FP8 element values fl32(e4m3 * scale), no BF16 intermediate).
 *   x          E4M3 [M_src, K], 16-byte aligned
 *   x_scale    FP32 [M_src, K/128], 4-byte aligned.  Blockwise FP8 carries finite positive scales; any other
 *              FP32 value acts through the IEEE-754 product: a NaN scale, or an infinite one times a zero
 *              element, makes the element NaN (block scale 0xFF, codes 0), an infinite one times a non-zero
 *              element overflows (block scale 254, code 7), a negative one flips the signs.
 *   gather_idx NULL: M_out must equal M_src and row i <- row i.
 *              else int32 [M_out] on the device: row i <- row gather_idx[i]
 *              (quantization placed right before the dispatch: the routing gather is fused).
 *   q          packed E2M1, M_out rows of K/2 bytes, row stride ld_q bytes (>= K/2);
 *              pointer and stride 8-byte aligned
 *   sf         UE8M0, M_out rows of K/32 bytes, row stride ld_sf bytes (>= K/32);
 *              pointer and stride 4-byte aligned
 * Dense outputs: ld_q = K/2, ld_sf = K/32.  One record per token (nibbles then scales):
 * ld_q = ld_sf = K/2 + K/32, sf = q + K/2. */
mxfp4_status mxfp4_quant_from_fp8(const uint8_t *x, const float *x_scale, int64_t M_src, int64_t K,
                                  const int32_t *gather_idx, int64_t M_out, uint8_t *q,
                                  int64_t ld_q, uint8_t *sf, int64_t ld_sf, void *hip_stream);

/* The same quantizer with the routing turned around (paper sec. 3.2: quantization sits right before
 * the dispatch): a token is read and quantized ONCE and its packed row written to each of its
 * destinations, instead of once per destination as with gather_idx.
 *   x, x_scale  as above, [M_src, K] and [M_src, K/128], dense
 *   dst_idx     int32 [M_src, fanout] on the device: source row i is written to the output rows
 *               dst_idx[i*fanout + j], j < fanout; an entry outside [0, M_out) is skipped.  Every
 *               output row may be named at most once (otherwise which copy it ends up holding is
 *               unspecified); output rows that no entry names keep their contents.
 *   q, ld_q, sf, ld_sf   M_out output rows, as above (planes or per-token records).  fanout >= 1. */
mxfp4_status mxfp4_quant_from_fp8_scatter(const uint8_t *x, const float *x_scale, int64_t M_src, int64_t K,
                                          const int32_t *dst_idx, int32_t fanout, int64_t M_out, uint8_t *q,
                                          int64_t ld_q, uint8_t *sf, int64_t ld_sf, void *hip_stream);

/* BF16 -> MXFP4: the row-wise quantizer as the paper states it (sec. 3.1, BF16ToFP4Row): the same
 * scale rule and rounding, applied to the BF16 values themselves.  NaN -> block scale 0xFF, codes 0;
 * +-inf -> block scale 254, code 7.
 *   x   BF16 bit patterns [M, K] dense, 16-byte aligned
 *   q   packed E2M1, row stride ld_q bytes (>= K/2); pointer and stride 4-byte aligned
 *   sf  UE8M0, row stride ld_sf bytes (>= K/32); pointer and stride 4-byte aligned */
mxfp4_status mxfp4_quant_from_bf16(const uint16_t *x, int64_t M, int64_t K, uint8_t *q, int64_t ld_q,
                                   uint8_t *sf, int64_t ld_sf, void *hip_stream);

/* MXFP4 -> FP8 (paper sec. 3.3, Algorithm 1: direct bit-wise remap with hierarchical scale
 * alignment).  Per 128-element tile with scale bytes b0..b3: the FP32 tile scale is
 * 2^(max(b) - 6 - 127), and every element becomes the E4M3 code of
 * e2m1(code) * 2^(6 - (max(b) - b_i)) -- the exponent re-bias of Algorithm 1 for normal
 * codes, rounding to nearest-even through the E4M3 subnormals when the alignment shift
 * pushes the exponent below 1.  Lossless when max(b) - b_i <= 14.
 *   q  [M, K/2] with row stride ld_q, 16-byte aligned pointer and stride
 *   sf [M, K/32] with row stride ld_sf
 *   x  E4M3 [M, K] dense, 16-byte aligned;  x_scale FP32 [M, K/128] dense, 4-byte aligned */
mxfp4_status mxfp4_dequant_to_fp8(const uint8_t *q, int64_t ld_q, const uint8_t *sf, int64_t ld_sf,
                                  int64_t M, int64_t K, uint8_t *x, float *x_scale,
                                  void *hip_stream);

/* Row-blocked MXFP4 -> column-blocked MXFP4 of the same matrix for the weight-gradient GEMM
 * (paper sec. 3.4: de-quantization, transposition and re-quantization fused in one pass
 * through on-chip memory).  Every element takes its exact value e2m1 * 2^(b_row - 127); each
 * run of 32 consecutive m at fixed k is re-quantized with the rule of sec. 3.1.
 *   q_row [M, K/2] dense, 4-byte aligned;  sf_row [M, K/32] dense, 4-byte aligned
 *   q_col [K, M/2] dense, 16-byte aligned; sf_col [K, M/32] dense
 *   M % 32 == 0; K at most 2^24. */
mxfp4_status mxfp4_row_to_col(const uint8_t *q_row, const uint8_t *sf_row, int64_t M, int64_t K,
                              uint8_t *q_col, uint8_t *sf_col, void *hip_stream);

/* Ragged per-expert forms (paper sec. 3.4, native support for ragged MoE tensors).
 *   expert_offsets  int32 [num_experts + 1] on the DEVICE: rows [off_e, off_{e+1}) belong to
 *                   expert e; off_0 = 0, off_E = M_total, non-decreasing; every
 *                   T_e = off_{e+1} - off_e may be ANY length >= 0 (no padding needed).
 *                   The pointer must be 4-byte aligned in every grouped form.
 * Quantization is row-independent, so the grouped form produces exactly what the flat form
 * produces on M_total rows (dense outputs); it checks the pointer and the count, and reads no offset.
 * Grouped row->column writes expert e as its own dense [K, ceil(T_e/2)] and [K, ceil(T_e/32)]
 * matrices at byte offsets K * sum_{j<e} ceil(T_j/2) of q_col and K * sum_{j<e} ceil(T_j/32) of
 * sf_col (= K*off_e/2 and K*off_e/32 when every T_e is a multiple of 32): contiguous storage
 * without padding.  No column block crosses an expert boundary; a last block of fewer than 32
 * rows is quantized over the rows it has, and with an odd T_e the unused high nibble of each
 * k-row's last byte is 0.  The buffers hold K * sum_e ceil(T_e/2) <= K * (M_total/2 + num_experts)
 * and K * sum_e ceil(T_e/32) <= K * (M_total/32 + num_experts) bytes. */
mxfp4_status mxfp4_quant_from_fp8_grouped(const uint8_t *x, const float *x_scale,
                                          const int32_t *expert_offsets, int32_t num_experts,
                                          int64_t M_total, int64_t K, uint8_t *q, uint8_t *sf,
                                          void *hip_stream);

mxfp4_status mxfp4_row_to_col_grouped(const uint8_t *q_row, const uint8_t *sf_row,
                                      const int32_t *expert_offsets, int32_t num_experts,
                                      int64_t M_total, int64_t K, uint8_t *q_col, uint8_t *sf_col,
                                      void *hip_stream);

/* Row-blocked MXFP4 -> the transposed matrix in FP8 for the weight-gradient GEMM (paper sec. 3.4,
 * the fused de-quantize / transpose / re-quantize kernel with FP8 output; the FP4 -> FP8 step is
 * the hierarchical scale alignment of sec. 3.3, Algorithm 1, taken along m).  For output row k and
 * each group of 128 consecutive rows m, with b_m = sf_row[m][k/32]:
 *   x_col_scale[k][m/128] = 2^(max(b) - 6 - 127)   (an FP32 subnormal when max(b) < 7)
 *   x_col[k][m]           = E4M3 code of e2m1(code[m][k]) * 2^(6 - (max(b) - b_m)),
 * rounded to nearest-even through the E4M3 subnormals; lossless while max(b) - b_m <= 14.
 * A 0xFF scale byte makes its group's scale NaN for the 32 k of its block and its own elements
 * 0x7F; the other rows align to the maximum of the non-NaN bytes.
 *   q_row [M, K/2] dense, 4-byte aligned;  sf_row [M, K/32] dense, 4-byte aligned
 *   x_col E4M3 [K, M] dense, 16-byte aligned;  x_col_scale FP32 [K, M/128] dense, 4-byte aligned
 *   M % 128 == 0; M and K at most 2^24. */
mxfp4_status mxfp4_row_to_fp8_col(const uint8_t *q_row, const uint8_t *sf_row, int64_t M, int64_t K,
                                  uint8_t *x_col, float *x_col_scale, void *hip_stream);

/* The same per expert, for ragged splits without padding (paper sec. 3.4): expert_offsets as above
 * but every T_e may be ANY length >= 0, and M_total need not be a multiple of 128.
 *   x_col        expert e's own dense [K, T_e] matrix at element offset K*off_e: contiguous storage
 *                without padding (rows of T_e bytes, so vector stores are unaligned when T_e % 16 != 0)
 *   x_col_scale  expert e's own dense [K, ceil(T_e/128)] matrix at element offset
 *                K * sum_{j<e} ceil(T_j/128) (= K*off_e/128 when every T_e is a multiple of 128);
 *                the buffer holds K * sum_e ceil(T_e/128) <= K * (M_total/128 + num_experts) floats.
 *                A last group of fewer than 128 rows takes its maximum over the rows it has.
 * No scale group crosses an expert boundary. */
mxfp4_status mxfp4_row_to_fp8_col_grouped(const uint8_t *q_row, const uint8_t *sf_row,
                                          const int32_t *expert_offsets, int32_t num_experts,
                                          int64_t M_total, int64_t K, uint8_t *x_col, float *x_col_scale,
                                          void *hip_stream);

/* The same two conversions under the other reading of the paper's fused kernel (sec. 3.4:
 * de-quantization, transposition and RE-QUANTIZATION, with the power-of-two scale
 * 2^ceil(log2 x) of its bit-level arithmetic item): every element takes its exact value
 * v = e2m1(code) * 2^(b_m - 127); per output row k and 128 consecutive m the scale is the smallest
 * power of two S with max|v| <= 448 * S (1.0 for an all-zero group, an FP32 subnormal below
 * 2^-126), and x_col[k][m] = E4M3 code of v / S, rounded to nearest-even.  Never a coarser scale
 * than the alignment form above, and the same bytes whenever the two scales coincide.
 * Arguments, layouts, limits and the NaN rule are those of mxfp4_row_to_fp8_col and
 * mxfp4_row_to_fp8_col_grouped (ragged splits of any length included). */
mxfp4_status mxfp4_row_to_fp8_col_requant(const uint8_t *q_row, const uint8_t *sf_row, int64_t M, int64_t K,
                                          uint8_t *x_col, float *x_col_scale, void *hip_stream);

mxfp4_status mxfp4_row_to_fp8_col_requant_grouped(const uint8_t *q_row, const uint8_t *sf_row,
                                                  const int32_t *expert_offsets, int32_t num_experts,
                                                  int64_t M_total, int64_t K, uint8_t *x_col,
                                                  float *x_col_scale, void *hip_stream);

/* Measurement aids, not conversions: byte movers without arithmetic.  The conversions are bandwidth-bound (the
 * paper places their cost in global-memory traffic, sec. 3.4 and 4.3), so their rates are reported beside what
 * a kernel reaches on the same GPU, in the same run, that only moves their bytes.
 *
 * mxfp4_stream_mix: `bytes` (a multiple of 16) bytes of the WIDER side, one 16-byte access per lane.
 *   mix 0  1:1 copy: src and dst of `bytes` bytes
 *   mix 1  2:1, the quantizer's mix: `bytes` read, bytes/2 written
 *   mix 2  1:2, the de-quantizer's mix: bytes/2 read, `bytes` written
 *   mix 3  read only: `bytes` read (dst must still be a valid pointer; one byte of it may be written)
 *   policy bit 0: non-temporal loads, bit 1: non-temporal stores (0..3)
 *   src, dst  device pointers, 16-byte aligned, not overlapping
 * mxfp4_stream_copy(src, dst, bytes, policy) is mix 0.
 *
 * mxfp4_tile_copy: the access pattern of the row->column conversions without the conversion.  src is a
 * row-major byte matrix [rows, row_bytes] (rows % 256 == 0, row_bytes % 128 == 0), dst the [2 * row_bytes,
 * rows / 2] byte matrix of the transposed nibble layout; every 256 x 128-byte tile of src is read with
 * 16-byte loads and written as 256 pieces of 128 bytes, piece i to row 256 * (tile column) + i of dst at
 * byte 128 * (tile row), in the tile order of the conversions.  The bytes inside a piece are not rearranged
 * (dst is not a transposition of src): it moves the nibble bytes mxfp4_row_to_col moves, where it moves them. */
mxfp4_status mxfp4_stream_copy(const void *src, void *dst, int64_t bytes, int32_t policy, void *hip_stream);
mxfp4_status mxfp4_stream_mix(const void *src, void *dst, int64_t bytes, int32_t policy, int32_t mix,
                              void *hip_stream);
mxfp4_status mxfp4_tile_copy(const void *src, void *dst, int64_t rows, int64_t row_bytes, void *hip_stream);

/* Measurement aid: the write traffic of mxfp4_quant_from_fp8_scatter without the quantizer.  Record i of src
 * (rec_bytes bytes at src + i * ld_src; rec_bytes a multiple of 16 up to 48 KiB, ld_src a multiple of 16) is
 * read once and written to the records dst_idx[i * fanout + j], j < fanout, of dst (record d at
 * dst + d * rec_bytes); entries outside [0, M_out) are skipped.  src, dst 16-byte aligned device pointers,
 * dst_idx int32 [M_src, fanout] on the device. */
mxfp4_status mxfp4_record_fanout(const void *src, int64_t ld_src, const int32_t *dst_idx, int64_t M_src,
                                 int32_t fanout, int64_t rec_bytes, int64_t M_out, void *dst, void *hip_stream);

/* Human-readable name of a status code (static storage, never NULL). */
const char *mxfp4_status_string(mxfp4_status status);

#ifdef __cplusplus
}
#endif

#endif /* MXFP4_H */
