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
#include "mxfp4_device.hpp"
#include "mxfp4_kernels.hpp"

namespace mxfp4 {

#ifndef MXFP4_F8C_PHASES
#define MXFP4_F8C_PHASES 2
#endif
#ifndef MXFP4_F8C_MBM
#define MXFP4_F8C_MBM 32
#endif
#ifndef MXFP4_F8C_MBK
#define MXFP4_F8C_MBK 4
#endif
#ifndef MXFP4_F8C_WAVES
#define MXFP4_F8C_WAVES 1
#endif

namespace fp8col {

constexpr int NRG = 8;              // 32-row groups per tile
constexpr int T_THREADS = 32 * NRG; // one lane per (row group, 8-column group)
constexpr int TILE_M = 32 * NRG;
constexpr int TILE_K = 256;
constexpr int PHASES = MXFP4_F8C_PHASES; // the tile leaves in PHASES parts of 8/PHASES columns per lane
constexpr int CP = 8 / PHASES;           // columns of a lane per phase
static_assert(PHASES == 1 || PHASES == 2 || PHASES == 4, "a phase is a whole number of nibble bytes");

typedef short s16x2 __attribute__((ext_vector_type(2)));

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
};

// Decode-scale operand of row I of a slice: exponent field max(127 - (bmax - b_I), 0) in bits
// 30:23, computed as a signed value so that one max() does the clamp.
template <int I>
__device__ __forceinline__ float row_shift_operand(const uint32_t (&sb)[8], int bias_minus_bmax)
{
    const int b = (int)((sb[I >> 2] >> (8 * (I & 3))) & 0xFFu);
    return u2f((uint32_t)max((int)((uint32_t)(b + bias_minus_bmax) << 23), 0));
}

// 0xFF in every byte of `bytes4` that equals 0xFF.
__device__ __forceinline__ uint32_t nan_byte_mask(uint32_t bytes4)
{
    const uint32_t top = ((bytes4 & 0x7F7F7F7Fu) + 0x01010101u) & bytes4 & 0x80808080u;
    return (top >> 7) * 0xFFu;
}

} // namespace fp8col

using namespace fp8col;

__global__ void __launch_bounds__(T_THREADS, MXFP4_F8C_WAVES) row_to_fp8_col_kernel(const Args a)
{
    __shared__ u32x4 s_out[(TILE_K / PHASES) * 16];      // [c'*32 + cg][16 slots]: k-rows of 256 B
    __shared__ alignas(16) uint8_t s_row_sf[8 * TILE_M]; // [k-block of the tile][row]
    __shared__ alignas(8) uint8_t s_max16[8 * 16];       // [k-block][16-row group]: max of the non-NaN bytes
    __shared__ uint8_t s_nan[4];                         // per wave: bit kb set = a NaN scale byte

    uint32_t tile_m, tile_k;
    if (!tile_of_workgroup<MXFP4_F8C_MBM, MXFP4_F8C_MBK>(blockIdx.x, a.tiles_m, a.tiles_k, &tile_m, &tile_k))
        return;

    // ---- which rows: the whole matrix, or one expert's slice (uniform per workgroup)
    uint32_t row_base = 0, rows = a.M;
    if (a.expert_offsets) {
        bool found = false;
        for (int e = 0; e < a.num_experts; ++e) {
            const uint32_t lo = (uint32_t)a.expert_offsets[e], hi = (uint32_t)a.expert_offsets[e + 1];
            const uint32_t nt = (hi - lo + TILE_M - 1) / TILE_M;
            if (tile_m < nt) {
                row_base = lo;
                rows = hi - lo;
                found = true;
                break;
            }
            tile_m -= nt;
        }
        if (!found)
            return;
    }
    const uint32_t m0 = tile_m * TILE_M; // first row of the tile inside its group
    if (m0 >= rows)
        return;
    const uint32_t n_rg = min((uint32_t)TILE_M, rows - m0) / 32u; // row groups present: 4 or 8
    const uint32_t n_g = n_rg / 4u;                              // 128-row scale groups present
    const uint32_t k0 = tile_k * TILE_K;
    const uint32_t cols = min((uint32_t)TILE_K, a.K - k0); // 128 or 256
    const uint32_t Kb = a.K / 32u;

    // expert e's output is its own dense [K, rows] and [K, rows/128]
    uint8_t *out_x = a.x_col + (size_t)a.K * row_base;
    float *out_s = a.x_col_scale + (size_t)a.K * row_base / 128u;
    const size_t pitch_x = rows, pitch_s = rows / 128u;

    const uint32_t tid = threadIdx.x;
    const uint32_t rg = tid >> 5, cg = tid & 31u;
    const uint32_t pitch = a.K / 2u;
    const bool active = rg < n_rg && cg * 8u < cols;

    // ---- the 32x8 slice of a lane: one dword (8 nibbles) per row
    uint32_t w[32];
    if (active) {
        const uint8_t *src = a.q_row + (size_t)(row_base + m0) * pitch + k0 / 2u + rg * 32u * pitch + cg * 4u;
#pragma unroll
        for (int i = 0; i < 32; ++i)
            w[i] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(src + (size_t)i * pitch));
    }

    // ---- stage the tile's row scales (thread t takes row t, 4 or 8 bytes) and reduce them:
    // per k-block the maximum of the non-NaN bytes over each 16 rows (DPP), and per wave
    // whether a NaN byte occurs.
    {
        uint32_t lo = 0, hi = 0;
        if (tid < n_rg * 32u) {
            const uint8_t *p = a.sf_row + (size_t)(row_base + m0 + tid) * Kb + k0 / 32u;
            if (cols > 128u && (reinterpret_cast<uintptr_t>(p) & 7u) == 0u) {
                const u32x2 v = *reinterpret_cast<const u32x2 *>(p);
                lo = v.x;
                hi = v.y;
            } else {
                lo = reinterpret_cast<const uint32_t *>(p)[0];
                hi = cols > 128u ? reinterpret_cast<const uint32_t *>(p)[1] : 0u;
            }
        }
        uint32_t nan_bits = 0, m_lo = 0, m_hi = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t b = ((j < 4 ? lo : hi) >> (8 * (j & 3))) & 0xFFu;
            s_row_sf[j * TILE_M + tid] = (uint8_t)b;
            nan_bits |= (__ballot(b == 255u) != 0ull ? 1u : 0u) << j;
            uint32_t v = b == 255u ? 0u : b;
            v = max(v, dpp_read<DPP_QUAD_XOR1>(v));
            v = max(v, dpp_read<DPP_QUAD_XOR2>(v));
            v = max(v, dpp_read<DPP_ROW_HALF_MIRROR>(v));
            v = max(v, dpp_read<DPP_ROW_MIRROR>(v));
            if (j < 4)
                m_lo |= v << (8 * j);
            else
                m_hi |= v << (8 * (j - 4));
        }
        if ((tid & 15u) == 0u) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                s_max16[j * 16 + (tid >> 4)] = (uint8_t)(m_lo >> (8 * j));
                s_max16[(4 + j) * 16 + (tid >> 4)] = (uint8_t)(m_hi >> (8 * j));
            }
        }
        if ((tid & 63u) == 0u)
            s_nan[tid >> 6] = (uint8_t)nan_bits;
    }
    __syncthreads();

    // ---- the lane's view: its k-block kb, its 128-row group g
    const uint32_t kb = cg >> 2, g = rg >> 2;
    uint32_t bmax;
    {
        const u32x2 p = *reinterpret_cast<const u32x2 *>(&s_max16[kb * 16 + g * 8]);
        uint32_t t = max(max(p.x & 0xFFu, (p.x >> 8) & 0xFFu), max((p.x >> 16) & 0xFFu, p.x >> 24));
        uint32_t u = max(max(p.y & 0xFFu, (p.y >> 8) & 0xFFu), max((p.y >> 16) & 0xFFu, p.y >> 24));
        bmax = max(t, u);
    }
    const bool has_nan = (((s_nan[2 * g] | s_nan[2 * g + 1]) >> kb) & 1u) != 0u;

    // ---- group scales: k-row t of the tile, one float per 128-row group
    if (tid < cols) {
        const uint32_t kbt = tid >> 5;
        uint32_t bits[2];
#pragma unroll
        for (int gg = 0; gg < 2; ++gg) {
            const u32x2 p = *reinterpret_cast<const u32x2 *>(&s_max16[kbt * 16 + gg * 8]);
            const uint32_t t = max(max(p.x & 0xFFu, (p.x >> 8) & 0xFFu), max((p.x >> 16) & 0xFFu, p.x >> 24));
            const uint32_t u = max(max(p.y & 0xFFu, (p.y >> 8) & 0xFFu), max((p.y >> 16) & 0xFFu, p.y >> 24));
            const int e = (int)max(t, u) - 6; // biased exponent of 2^(max - 6 - 127); below 1: an FP32 subnormal
            bits[gg] = e >= 1 ? (uint32_t)e << 23 : 0x00400000u >> (uint32_t)(-e);
            if ((((s_nan[2 * gg] | s_nan[2 * gg + 1]) >> kbt) & 1u) != 0u)
                bits[gg] = 0x7FC00000u;
        }
        float *dst = out_s + (size_t)(k0 + tid) * pitch_s + m0 / 128u;
        if (n_g == 2u && (reinterpret_cast<uintptr_t>(dst) & 7u) == 0u) {
            *reinterpret_cast<u32x2 *>(dst) = u32x2{bits[0], bits[1]};
        } else {
            if (n_g >= 1u)
                dst[0] = u2f(bits[0]);
            if (n_g == 2u)
                dst[1] = u2f(bits[1]);
        }
    }

    // ---- the 32 row-scale bytes of this slice (byte i%4 of dword i/4 is row i) -> decode operands
    uint32_t sb[8];
    float dsc[32];
    if (active) {
        const uint8_t *my_row_sf = &s_row_sf[kb * TILE_M + rg * 32u];
        const u32x4 s0 = reinterpret_cast<const u32x4 *>(my_row_sf)[0];
        const u32x4 s1 = reinterpret_cast<const u32x4 *>(my_row_sf)[1];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            sb[q] = s0[q];
            sb[4 + q] = s1[q];
        }
        const int bias_minus_bmax = 127 - (int)bmax;
        static_for<32>([&](auto ip) {
            constexpr int i = decltype(ip)::value;
            dsc[i] = row_shift_operand<i>(sb, bias_minus_bmax);
        });
    }
    const float enc = u2f(121u << 23); // the encoder divides by 2^-6: Algorithm 1's delta

    const uint32_t slot0 = (2u * rg + cg) & 15u; // 16-byte slots of rows 0..15 / 16..31 of the slice
    const uint32_t slot1 = (2u * rg + 1u + cg) & 15u;

    static_for<PHASES>([&](auto php) {
        constexpr int ph = decltype(php)::value;
        if (active) {
            static_for<CP / 2>([&](auto jjp) {
                constexpr int j = ph * (CP / 2) + decltype(jjp)::value; // nibble byte: columns 2j, 2j+1
                uint32_t o[2][8];
                static_for<8>([&](auto rp) {
                    constexpr int r = decltype(rp)::value; // rows 4r..4r+3 -> dword r of both columns
                    const f32x2 f0 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[4 * r], dsc[4 * r], j);
                    const f32x2 f1 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[4 * r + 1], dsc[4 * r + 1], j);
                    const f32x2 f2 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[4 * r + 2], dsc[4 * r + 2], j);
                    const f32x2 f3 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[4 * r + 3], dsc[4 * r + 3], j);
                    s16x2 e0 = {0, 0}, e1 = {0, 0};
                    e0 = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(e0, f0.x, f1.x, enc, false);
                    e0 = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(e0, f2.x, f3.x, enc, true);
                    e1 = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(e1, f0.y, f1.y, enc, false);
                    e1 = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(e1, f2.y, f3.y, enc, true);
                    o[0][r] = __builtin_bit_cast(uint32_t, e0);
                    o[1][r] = __builtin_bit_cast(uint32_t, e1);
                    if (has_nan) { // rare: rows under a NaN scale byte become E4M3 NaN
                        const uint32_t nm = nan_byte_mask(sb[r]);
                        o[0][r] = (o[0][r] & ~nm) | (0x7F7F7F7Fu & nm);
                        o[1][r] = (o[1][r] & ~nm) | (0x7F7F7F7Fu & nm);
                    }
                });
#pragma unroll
                for (int cc = 0; cc < 2; ++cc) {
                    const uint32_t row = ((2 * j + cc) - ph * CP) * 32u + cg; // LDS k-row of column 2j+cc
                    s_out[row * 16u + slot0] = u32x4{o[cc][0], o[cc][1], o[cc][2], o[cc][3]};
                    s_out[row * 16u + slot1] = u32x4{o[cc][4], o[cc][5], o[cc][6], o[cc][7]};
                }
            });
        }
        __syncthreads();

        // ---- write the part out: 16 lanes per k-row, 256 contiguous bytes.  Chunk u*256 + tid of
        // the LDS part is row u*16 + tid/16 = c'*32 + cgx, physical slot tid%16.
        {
            const uint32_t pslot = tid & 15u;
#pragma unroll
            for (int u = 0; u < 2 * CP; ++u) {
                const uint32_t cgx = (u & 1) * 16u + (tid >> 4);
                const uint32_t c = ph * CP + (u >> 1);
                const uint32_t lslot = (pslot - cgx) & 15u; // 16 bytes = rows 16*lslot.. of the tile
                if (cgx * 8u < cols && (lslot >> 1) < n_rg) {
                    uint8_t *dst = out_x + (size_t)(k0 + cgx * 8u + c) * pitch_x + m0 + lslot * 16u;
                    *reinterpret_cast<u32x4 *>(dst) = s_out[u * T_THREADS + tid];
                }
            }
        }
        if (ph + 1 < PHASES)
            __syncthreads(); // the LDS part is free again
    });
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
    const dim3 grid((total + NUM_XCD - 1) / NUM_XCD * NUM_XCD);
    hipLaunchKernelGGL(row_to_fp8_col_kernel, grid, dim3(T_THREADS), 0, stream, a);
    return hipGetLastError();
}

} // namespace mxfp4
