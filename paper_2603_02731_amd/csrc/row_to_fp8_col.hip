// Row-blocked MXFP4 -> the transposed matrix as FP8 (E4M3 [K,M] + FP32 scale per 128 m), gfx950.
//
// Paper sec. 3.4: the weight-gradient GEMM needs the transposed activations in FP8, and
// de-quantization, transposition and re-quantization are fused into one pass through on-chip
// memory.  The FP4 -> FP8 step is the hierarchical scale alignment of sec. 3.3 (Algorithm 1)
// taken along m: for output row k and 128 consecutive rows m with scale bytes
// b_m = sf_row[m][k/32], the group scale is 2^(max(b) - 6 - 127) and the element is
// e2m1 * 2^(6 - (max(b) - b_m)) as E4M3 (exact while the shift is at most 14, rounded to
// nearest-even through the E4M3 subnormals beyond, zero from 19).
//
// Work split: as in the MXFP4 -> MXFP4 transposing kernel, a workgroup of 256 lanes owns a
// 256 (m) x 256 (k) tile and lane (rg, cg) the rows 32*rg.. and the columns 8*cg.., i.e. 32
// dwords of nibbles.  Everything is relative to the group maximum, so no value leaves FP32:
//   v_cvt_scalef32_pk_f32_fp4 decodes two columns of a row with the scale operand
//       2^-(max(b) - b_m)  (exponent field 127 - shift, clamped at 0: far below E4M3 anyway),
//   v_cvt_scalef32_pk_fp8_f32 takes the values of rows (m, m+1) of one column, divides by
//       2^-6 and rounds onto E4M3; two of them fill a dword of four consecutive m.
// The register pairing is the transposition.  The per-group maxima come from the staged row
// scales: a 16-lane DPP reduction per k-block while staging, finished after the barrier.
// The 8 x 32 B of a lane leave through an LDS tile whose 16-byte slots are rotated by the
// column group (conflict-free writes, linear read-back) as full 256-byte rows.
#include "fp8_col_tile.hpp"
#include "mxfp4_device.hpp"
#include "mxfp4_kernels.hpp"

namespace mxfp4 {

// Macro block of the tile order: 4 column tiles; row tiles by macro_block_rows for one matrix (32 at [65536,7168]:
// over rotated buffers 127.5 us, 16 x 4 129 us, 8 x 4 164 us; 2 or 8 k-tiles: no difference; [61440,7168] 146 -> 124 us
// against a fixed 32), at most MBM_MAX inside an expert (on experts of 512 to 4096 rows, whose macro blocks end with
// the expert, 16 and 32 row tiles are equally fast).  Measured and not built: a lane owning 16 rows with 512 lanes per
// tile (142 us), the tile leaving in 2 or 4 LDS passes for more workgroups per CU (146-162 us), k-fastest tile order
// (144 us), plain instead of non-temporal stores for the 256-byte output rows (145 us over rotated buffers).
namespace fp8col {

constexpr uint32_t MBM_MAX = 64, MBK = 4; // macro block of the tile order
constexpr int RPL = 32;              // rows of a lane's slice
constexpr int TILE_M = 256;
constexpr int TILE_K = 256;
constexpr int T_THREADS = 32 * (TILE_M / RPL); // one lane per (row group, 8-column group)
constexpr int SPL = RPL / 16;        // 16-byte output slots of a lane per column

struct Args {
    const uint8_t *q_row;
    const uint8_t *sf_row;
    uint8_t *x_col;
    float *x_col_scale;
    const int32_t *expert_offsets; // nullptr: one group of M rows
    int32_t num_experts;
    uint32_t M;
    uint32_t K;
    uint32_t tiles_m; // 256-row tiles (an upper bound when grouped)
    uint32_t tiles_k; // 256-column tiles
    uint32_t stage_in; // full tiles fetch their nibbles with 16-byte loads and re-slice them through LDS
    uint32_t mbm;      // row tiles per macro block of the tile order (one matrix; experts: see the lookup)
};

// Decode-scale operand of row I of a slice: exponent field max(127 - (bmax - b_I), 0) in bits
// 30:23, computed as a signed value so that one max() does the clamp.
template <int I>
__device__ __forceinline__ float row_shift_operand(const uint32_t (&sb)[RPL / 4], int bias_minus_bmax)
{
    const int b = (int)((sb[I >> 2] >> (8 * (I & 3))) & 0xFFu);
    return u2f((uint32_t)max((int)((uint32_t)(b + bias_minus_bmax) << 23), 0));
}

// Maximum of the 8 bytes at p (8-byte aligned, LDS).
__device__ __forceinline__ uint32_t max_of_8_bytes(const uint8_t *p)
{
    const u32x2 v = *reinterpret_cast<const u32x2 *>(p);
    const uint32_t t = max(max(v.x & 0xFFu, (v.x >> 8) & 0xFFu), max((v.x >> 16) & 0xFFu, v.x >> 24));
    const uint32_t u = max(max(v.y & 0xFFu, (v.y >> 8) & 0xFFu), max((v.y >> 16) & 0xFFu, v.y >> 24));
    return max(t, u);
}

} // namespace fp8col

using namespace fp8col;

__global__ void __launch_bounds__(T_THREADS) row_to_fp8_col_kernel(const Args a)
{
    __shared__ u32x4 s_out[TILE_K * 16];                 // [c*32 + cg][16 slots]: k-rows of 256 B
    __shared__ alignas(16) uint8_t s_row_sf[8 * TILE_M]; // [k-block of the tile][row]
    __shared__ alignas(8) uint8_t s_max16[8 * 16];       // [k-block][16-row group]: max of the non-NaN bytes
    __shared__ uint8_t s_nan[4 * 8];                     // [64-row group][k-block]: a NaN scale byte occurs

    // ---- which tile, and which rows: the whole matrix, or one expert's slice of any length (uniform
    // per workgroup)
    uint32_t tile_m, tile_k;
    uint32_t row_base = 0, rows = a.M, groups_before = 0;
    if (a.expert_offsets) {
        if (!tile_of_grouped_workgroup<TILE_M, 128, 0, MBM_MAX, MBK>(a.expert_offsets, a.num_experts, blockIdx.x, a.tiles_k,
                                                                 &tile_m, &tile_k, &row_base, &rows, &groups_before))
            return;
    } else if (!tile_of_workgroup<MBK>(blockIdx.x, a.tiles_m, a.tiles_k, a.mbm, &tile_m, &tile_k)) {
        return;
    }
    const uint32_t m0 = tile_m * TILE_M; // first row of the tile inside its group
    if (m0 >= rows)
        return;
    const uint32_t n_rows = min((uint32_t)TILE_M, rows - m0); // rows present: 1..256
    const uint32_t n_g = (n_rows + 127u) / 128u;              // scale groups present, the last maybe partial
    const uint32_t k0 = tile_k * TILE_K;
    const uint32_t cols = min((uint32_t)TILE_K, a.K - k0); // 128 or 256
    const uint32_t Kb = a.K / 32u;

    // expert e's output is its own dense [K, rows] and [K, ceil(rows/128)], the latter after the
    // scale groups of the experts before it
    uint8_t *out_x = a.x_col + (size_t)a.K * row_base;
    float *out_s = a.x_col_scale + (size_t)a.K * (a.expert_offsets ? groups_before : 0u);
    const size_t pitch_x = rows, pitch_s = (rows + 127u) / 128u;

    const uint32_t tid = threadIdx.x;
    const uint32_t rgl = tid >> 5, cg = tid & 31u;
    const uint32_t pitch = a.K / 2u;
    const bool active = rgl * RPL < n_rows && cg * 8u < cols;

    // ---- the RPL x 8 slice of a lane: one dword (8 nibbles) per row, from a uniform row pointer
    // plus a 32-bit lane offset (one address register, not RPL pairs)
    uint32_t w[RPL];
    // On grids with many tiles per CU (flat or per-expert) a full tile arrives through 16-byte loads (8 rows x 128 bytes per
    // wave instruction instead of 2) and is cut into the lanes' slices through the tile buffer, behind one
    // more barrier: 133.6 -> 127.0 us at [65536,7168] launched back to back, 200 -> 190 us over 32 un-padded experts.
    const bool staged = a.stage_in != 0u && n_rows == (uint32_t)TILE_M &&
                        cols == (uint32_t)TILE_K && (reinterpret_cast<uintptr_t>(a.q_row) & 15u) == 0u;
    u32x4 stage_v[8];
    if (staged) {
        const uint32_t wv = tid >> 6, lane = tid & 63u;
        const uint8_t *src = a.q_row + (size_t)(row_base + m0) * pitch + k0 / 2u +
                             (size_t)(wv * 64u + (lane >> 3)) * pitch + (lane & 7u) * 16u;
#pragma unroll
        for (int j = 0; j < 8; ++j)
            stage_v[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + (size_t)(j * 8) * pitch));
    } else if (active) {
        const uint8_t *tile_src = a.q_row + (size_t)(row_base + m0) * pitch + k0 / 2u;
        const uint32_t lane_off = rgl * RPL * pitch + cg * 4u; // < 2^32: K is at most 2^24
        if (n_rows == (uint32_t)TILE_M) {
#pragma unroll
            for (int i = 0; i < RPL; ++i)
                w[i] = __builtin_nontemporal_load(
                    reinterpret_cast<const uint32_t *>(tile_src + (size_t)i * pitch + lane_off));
        } else {
            // ragged end of a split: rows past it are read from its last row instead (their
            // results are never stored and their scale bytes are staged as 0)
            const uint32_t last = n_rows - 1u - rgl * RPL;
#pragma unroll
            for (int i = 0; i < RPL; ++i)
                w[i] = __builtin_nontemporal_load(
                    reinterpret_cast<const uint32_t *>(tile_src + lane_off + min((uint32_t)i, last) * pitch));
        }
    }

    // ---- stage the tile's row scales (thread t takes row t, 8 bytes) and reduce them:
    // per k-block the maximum of the non-NaN bytes over each 16 rows (DPP), and per 64 rows
    // (a wave) whether a NaN byte occurs.
    {
        const uint32_t row = tid;
        uint32_t v[2] = {0u, 0u};
        if (row < n_rows) {
            const uint8_t *p = a.sf_row + (size_t)(row_base + m0 + row) * Kb + k0 / 32u;
            if (cols > 128u) { // one request at any 4-byte alignment
                const u32x2 t = *reinterpret_cast<const u32x2_unaligned *>(p);
                v[0] = t.x;
                v[1] = t.y;
            } else {
                v[0] = reinterpret_cast<const uint32_t *>(p)[0];
            }
        }
        uint32_t mx[2] = {0u, 0u}, nan_bits = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t b = (v[j >> 2] >> (8 * (j & 3))) & 0xFFu;
            s_row_sf[j * TILE_M + row] = (uint8_t)b;
            nan_bits |= (__ballot(b == 255u) != 0ull ? 1u : 0u) << j;
            uint32_t t = b == 255u ? 0u : b;
            t = max(t, dpp_read<DPP_QUAD_XOR1>(t));
            t = max(t, dpp_read<DPP_QUAD_XOR2>(t));
            t = max(t, dpp_read<DPP_ROW_HALF_MIRROR>(t));
            t = max(t, dpp_read<DPP_ROW_MIRROR>(t));
            mx[j >> 2] |= t << (8 * (j & 3));
        }
        if ((tid & 15u) == 0u) {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                s_max16[j * 16 + (row >> 4)] = (uint8_t)(mx[j >> 2] >> (8 * (j & 3)));
        }
        if ((tid & 63u) == 0u) {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                s_nan[(row >> 6) * 8 + j] = (uint8_t)((nan_bits >> j) & 1u);
        }
    }
    if (staged) {
        const uint32_t wv = tid >> 6, lane = tid & 63u;
#pragma unroll
        for (int j = 0; j < 8; ++j)
            s_out[(wv * 64u + j * 8u) * 8u + lane] = stage_v[j];
    }
    __syncthreads();
    if (staged) {
        const uint32_t *s_in = reinterpret_cast<const uint32_t *>(s_out) + rgl * 32u * 32u + cg;
#pragma unroll
        for (int i = 0; i < RPL; ++i)
            w[i] = s_in[i * 32];
        __syncthreads(); // every slice is in registers before the tile buffer takes the results
    }

    // ---- the lane's view: its k-block kb, its 128-row group g
    const uint32_t kb = cg >> 2, g = (rgl * RPL) >> 7;
    const uint32_t bmax = max_of_8_bytes(&s_max16[kb * 16 + g * 8]);
    const bool has_nan = (s_nan[(2 * g) * 8 + kb] | s_nan[(2 * g + 1) * 8 + kb]) != 0u;

    // ---- group scales: k-row t of the tile, one float per 128-row group
    if (tid < cols) {
        const uint32_t kbt = tid >> 5;
        uint32_t bits[2];
#pragma unroll
        for (int gg = 0; gg < 2; ++gg) {
            // biased exponent of 2^(max - 6 - 127); below 1: an FP32 subnormal
            const int e = (int)max_of_8_bytes(&s_max16[kbt * 16 + gg * 8]) - 6;
            bits[gg] = e >= 1 ? (uint32_t)e << 23 : 0x00400000u >> (uint32_t)(-e);
            if ((s_nan[(2 * gg) * 8 + kbt] | s_nan[(2 * gg + 1) * 8 + kbt]) != 0u)
                bits[gg] = 0x7FC00000u;
        }
        float *dst = out_s + (size_t)(k0 + tid) * pitch_s + m0 / 128u;
        // one request per k-row: an expert's scale rows start at any multiple of 4 bytes
        if (n_g == 2u)
            *reinterpret_cast<u64_unaligned *>(dst) = ((uint64_t)bits[1] << 32) | bits[0];
        else if (n_g == 1u)
            dst[0] = u2f(bits[0]);
    }

    // ---- the row-scale bytes of this slice (byte i%4 of dword i/4 is row i) -> decode operands
    uint32_t sb[RPL / 4];
    float dsc[RPL];
    const uint8_t *my_row_sf = &s_row_sf[kb * TILE_M + rgl * RPL];
    if (active) {
#pragma unroll
        for (int h = 0; h < SPL; ++h) {
            const u32x4 t = reinterpret_cast<const u32x4 *>(my_row_sf)[h];
#pragma unroll
            for (int q = 0; q < 4; ++q)
                sb[4 * h + q] = t[q];
        }
        const int bias_minus_bmax = 127 - (int)bmax;
        static_for<RPL>([&](auto ip) {
            constexpr int i = decltype(ip)::value;
            dsc[i] = row_shift_operand<i>(sb, bias_minus_bmax);
        });
    }
    const float enc = u2f(121u << 23); // the encoder divides by 2^-6: Algorithm 1's delta

    // 16-byte slot h of the slice (its rows 16h..16h+15) goes to physical slot (logical + cg) % 16
    uint32_t slot[SPL];
#pragma unroll
    for (int h = 0; h < SPL; ++h)
        slot[h] = (rgl * SPL + h + cg) & 15u;

    {
        if (active) {
            static_for<4>([&](auto jjp) {
                constexpr int j = decltype(jjp)::value; // nibble byte: columns 2j, 2j+1
                uint32_t o[2][RPL / 4];
                static_for<RPL / 4>([&](auto rp) {
                    constexpr int r = decltype(rp)::value; // rows 4r..4r+3 -> dword r of both columns
                    const f32x2 f0 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[4 * r], dsc[4 * r], j);
                    const f32x2 f1 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[4 * r + 1], dsc[4 * r + 1], j);
                    const f32x2 f2 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[4 * r + 2], dsc[4 * r + 2], j);
                    const f32x2 f3 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[4 * r + 3], dsc[4 * r + 3], j);
                    s16x2 e0, e1; // no initial value needed: both words are written
                    asm volatile("" : "=v"(e0), "=v"(e1));
                    e0 = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(e0, f0.x, f1.x, enc, false);
                    e0 = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(e0, f2.x, f3.x, enc, true);
                    e1 = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(e1, f0.y, f1.y, enc, false);
                    e1 = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(e1, f2.y, f3.y, enc, true);
                    o[0][r] = __builtin_bit_cast(uint32_t, e0);
                    o[1][r] = __builtin_bit_cast(uint32_t, e1);
                });
#pragma unroll
                for (int cc = 0; cc < 2; ++cc) {
                    const uint32_t row = (2 * j + cc) * 32u + cg; // LDS k-row of column 2j+cc
#pragma unroll
                    for (int h = 0; h < SPL; ++h)
                        s_out[row * 16u + slot[h]] =
                            u32x4{o[cc][4 * h], o[cc][4 * h + 1], o[cc][4 * h + 2], o[cc][4 * h + 3]};
                }
            });
            if (has_nan) {
                // rare: the rows under a NaN scale byte become E4M3 NaN; patched byte by byte in the
                // lane's own LDS slots (rolled: this path is written for size, not speed)
                uint8_t *bytes = reinterpret_cast<uint8_t *>(s_out);
#pragma nounroll
                for (uint32_t i = 0; i < (uint32_t)RPL; ++i) {
                    if (my_row_sf[i] != 255u)
                        continue;
                    const uint32_t sl = (rgl * SPL + (i >> 4) + cg) & 15u;
#pragma nounroll
                    for (uint32_t c = 0; c < 8u; ++c)
                        bytes[((c * 32u + cg) * 16u + sl) * 16u + (i & 15u)] = 0x7Fu;
                }
            }
        }
        __syncthreads();

        write_tile_out(s_out, out_x + (size_t)k0 * pitch_x + m0, out_x, pitch_x, cols, n_rows, tid);
    }
}

hipError_t launch_row_to_fp8_col(const uint8_t *q_row, const uint8_t *sf_row, const int32_t *expert_offsets,
                                 int32_t num_experts, int64_t M, int64_t K, uint8_t *x_col, float *x_col_scale,
                                 hipStream_t stream)
{
    Args a;
    a.q_row = q_row;
    a.sf_row = sf_row;
    a.x_col = x_col;
    a.x_col_scale = x_col_scale;
    a.expert_offsets = expert_offsets;
    a.num_experts = num_experts;
    a.M = (uint32_t)M;
    a.K = (uint32_t)K;
    // upper bound on the number of row tiles: every expert may end in a partial one
    a.tiles_m = (uint32_t)((M + TILE_M - 1) / TILE_M + (expert_offsets ? num_experts : 0));
    a.tiles_k = (uint32_t)((K + TILE_K - 1) / TILE_K);
    const uint32_t total = a.tiles_m * a.tiles_k;
    // at least 4 tiles per compute unit (over rotated buffers: 3-5 % slower at 640 to 896 tiles, 1-4 % faster from 1024 on)
    a.stage_in = total >= 4u * compute_units() ? 1u : 0u;
    a.mbm = macro_block_rows(a.tiles_m);
    const dim3 grid((total + NUM_XCD - 1) / NUM_XCD * NUM_XCD);
    hipLaunchKernelGGL(row_to_fp8_col_kernel, grid, dim3(T_THREADS), 0, stream, a);
    return hipGetLastError();
}

} // namespace mxfp4
