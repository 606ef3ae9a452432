// Row-blocked MXFP4 -> the transposed matrix as FP8 by re-quantization, gfx950.
//
// Paper sec. 3.4 read literally: de-quantize, transpose, re-quantize, with the power-of-two scale
// 2^ceil(log2 x) of its bit-level arithmetic item.  For output row k and 128 consecutive rows m
// the elements take their exact values v_m = e2m1 * 2^(b_m - 127); the group scale is the
// smallest power of two S with max|v| <= 448 * S (1.0 for an all-zero group); the element is
// v_m / S rounded to nearest-even E4M3.
//
// The scale in integers.  A non-zero E2M1 value is (1 + M/2) * 2^(E-1) with E its exponent field
// (0.5 = 2^-1: E = 0), and 448 = 1.75 * 2^8 lies between 1.5 and 2 times a power of two, so
// ceil(log2(v/448)) = floor(log2 v) - 8 and S = 2^(Emax - 136), Emax = max(b_m + E_m) over the
// non-zero codes: exactly the biased FP32 exponent of max|v| plus one, minus 136.
//
// Work split: the 256 x 256 tile and the 32 x 8 lane slices of the other transposing kernels.
//   pass 1: v_cvt_scalef32_pk_f32_fp4 with the row scale, running |max| per column; the four
//           lanes that share a column of a 128-row group exchange their maxima through LDS.
//   pass 2: decode again; v_cvt_scalef32_pk_fp8_f32 takes rows (m, m+1) of one column and divides
//           by 2^(Emax - 136), given as the operand exponent Emax - 9.
// Exact while every v is an FP32 number (row-scale bytes up to 252) and the operand exponent is
// not negative (Emax >= 9).  Lanes that see a byte of 253 or more (beyond FP32, or NaN) in their
// group, or a column maximum below 2^-118, take an integer path instead; neither occurs in real
// activations, so that path is written for size.
#include "fp8_col_tile.hpp"
#include "mxfp4_device.hpp"
#include "mxfp4_kernels.hpp"

namespace mxfp4 {

namespace fp8col_requant {

using namespace fp8col;

constexpr int TILE_M = 256, TILE_K = 256, T_THREADS = 256;

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

// Emax = biased exponent of a non-zero column maximum, plus one (FP32 subnormals: 2^-127 and
// 1.5 * 2^-127 give 1, 2^-128 gives 0).
__device__ __forceinline__ int emax_of_amax_bits(uint32_t bits)
{
    const int ef = (int)(bits >> 23);
    return ef >= 1 ? ef + 1 : (bits >= 0x00400000u ? 1 : 0);
}

// FP32 bit pattern of the group scale 2^(Emax - 136) (an FP32 subnormal for Emax <= 9); 1.0 for
// a group without a non-zero element.
__device__ __forceinline__ uint32_t scale_bits_of_emax(int emax, bool any_nonzero)
{
    if (!any_nonzero)
        return 0x3F800000u;
    const int field = emax - 9;
    return field >= 1 ? (uint32_t)field << 23 : 0x00400000u >> (uint32_t)(-field);
}

// The integer path.  Column kc of the tile over the rows [r0, r0 + n) of the tile (one scale
// group): Emax over the non-zero codes of the rows whose scale byte is not NaN, or -1 without
// any, plus GROUP_HAS_NAN when a NaN byte occurs.  Nibbles come from global memory, scale bytes
// from the staged copy.
constexpr int GROUP_HAS_NAN = 1 << 16;
__device__ __noinline__ int group_emax_int(const uint8_t *tile_src, size_t pitch, const uint8_t *row_sf_kb,
                                           uint32_t kc, uint32_t r0, uint32_t n)
{
    int emax = -1;
    bool any_nan = false;
#pragma nounroll
    for (uint32_t r = r0; r < r0 + n; ++r) {
        const uint32_t b = row_sf_kb[r];
        const uint32_t byte = tile_src[(size_t)r * pitch + (kc >> 1)];
        const uint32_t mag = ((kc & 1u) ? byte >> 4 : byte) & 7u;
        if (b == 255u)
            any_nan = true;
        else if (mag)
            emax = max(emax, (int)b + (int)(mag >> 1));
    }
    return emax + (any_nan ? GROUP_HAS_NAN : 0);
}

// E4M3 byte of +-e2m1(nib) * 2^(b - 127) / 2^(emax - 136) in integers.  With h = 2 * |e2m1| the
// quotient is h * 2^(b - emax + 17) quanta of 2^-9 (the E4M3 subnormal step): an exact integer n
// when the shift is not negative, else rounded to nearest-even; n < 16 is its own code
// (subnormals and the first binade), above that the binade is the position of the leading bit.
__device__ __forceinline__ uint32_t e4m3_requant_int(uint32_t nib, uint32_t b, int emax)
{
    const uint32_t mag = nib & 7u, sign = (nib & 8u) << 4;
    const uint32_t h = mag < 4u ? mag : mag == 4u ? 4u : mag == 5u ? 6u : mag == 6u ? 8u : 12u;
    if (mag == 0u)
        return sign;
    const int sh = (int)b - emax + 17;
    uint32_t n;
    if (sh >= 0) {
        n = h << sh;
    } else if (sh < -5) {
        n = 0;
    } else {
        const uint32_t t = (uint32_t)(-sh), q = h >> t, rem = h & ((1u << t) - 1u), half = 1u << (t - 1u);
        n = q + ((rem > half || (rem == half && (q & 1u))) ? 1u : 0u);
    }
    if (n < 16u)
        return sign | n;
    const uint32_t p = 31u - (uint32_t)__builtin_clz(n);
    return sign | ((p - 2u) << 3) | ((n >> (p - 3u)) & 7u);
}

} // namespace fp8col_requant

using namespace fp8col_requant;

__global__ void __launch_bounds__(T_THREADS) row_to_fp8_col_requant_kernel(const fp8col_requant::Args a)
{
    __shared__ u32x4 s_out[TILE_K * 16];                 // [c*32 + cg][16 slots]: k-rows of 256 B
    __shared__ alignas(16) uint8_t s_row_sf[8 * TILE_M]; // [k-block of the tile][row]
    __shared__ alignas(16) float s_amax[8 * TILE_K];     // [32-row group][column]: maxima of pass 1
    __shared__ uint8_t s_special[4 * 8];                 // [64-row group][k-block]: a scale byte >= 253

    // ---- which tile, and which rows: the whole matrix, or one expert's slice of any length (uniform
    // per workgroup)
    uint32_t tile_m, tile_k;
    uint32_t row_base = 0, rows = a.M, groups_before = 0;
    if (a.expert_offsets) {
        if (!tile_of_grouped_workgroup<TILE_M, 128, 0, 64, 4>(a.expert_offsets, a.num_experts, blockIdx.x, a.tiles_k,
                                                              &tile_m, &tile_k, &row_base, &rows, &groups_before))
            return;
    } else if (!tile_of_workgroup<4>(blockIdx.x, a.tiles_m, a.tiles_k, a.mbm, &tile_m, &tile_k)) {
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
    const uint32_t rg = tid >> 5, cg = tid & 31u;
    const uint32_t pitch = a.K / 2u;
    const bool in_cols = cg * 8u < cols;
    const bool active = rg * 32u < n_rows && in_cols;
    const uint8_t *tile_src = a.q_row + (size_t)(row_base + m0) * pitch + k0 / 2u;

    // ---- the 32x8 slice of a lane: one dword (8 nibbles) per row
    uint32_t w[32];
    // On grids with many tiles per CU (flat or per-expert) a full tile arrives through 16-byte loads (8 rows x 128 bytes per
    // wave instruction instead of 2) and is cut into the lanes' slices through the tile buffer, behind one
    // more barrier.
    const bool staged = a.stage_in != 0u && n_rows == (uint32_t)TILE_M && cols == (uint32_t)TILE_K &&
                        (reinterpret_cast<uintptr_t>(a.q_row) & 15u) == 0u;
    u32x4 stage_v[8];
    if (staged) {
        const uint32_t wv = tid >> 6, lane = tid & 63u;
        const uint8_t *src = tile_src + (size_t)(wv * 64u + (lane >> 3)) * pitch + (lane & 7u) * 16u;
#pragma unroll
        for (int j = 0; j < 8; ++j)
            stage_v[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + (size_t)(j * 8) * pitch));
    } else if (active) {
        const uint32_t lane_off = rg * 32u * pitch + cg * 4u; // < 2^32: K is at most 2^24
        if (n_rows == (uint32_t)TILE_M) {
#pragma unroll
            for (int i = 0; i < 32; ++i)
                w[i] = __builtin_nontemporal_load(
                    reinterpret_cast<const uint32_t *>(tile_src + (size_t)i * pitch + lane_off));
        } else {
            // ragged end of a split: rows past it count as zeros (read from the last row, then cleared)
            const uint32_t last = n_rows - 1u - rg * 32u;
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                const uint32_t v = __builtin_nontemporal_load(
                    reinterpret_cast<const uint32_t *>(tile_src + lane_off + min((uint32_t)i, last) * pitch));
                w[i] = (uint32_t)i <= last ? v : 0u;
            }
        }
    }

    // ---- stage the tile's row scales: thread t takes row t, 4 or 8 bytes; one ballot per k-block
    // tells which (64-row group, k-block) pairs hold a byte of 253 or more
    {
        uint32_t lo = 0, hi = 0;
        if (tid < n_rows) {
            const uint8_t *p = a.sf_row + (size_t)(row_base + m0 + tid) * Kb + k0 / 32u;
            if (cols > 128u) { // one request at any 4-byte alignment
                const u32x2 v = *reinterpret_cast<const u32x2_unaligned *>(p);
                lo = v.x;
                hi = v.y;
            } else {
                lo = reinterpret_cast<const uint32_t *>(p)[0];
            }
        }
        uint32_t special = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t b = ((j < 4 ? lo : hi) >> (8 * (j & 3))) & 0xFFu;
            s_row_sf[j * TILE_M + tid] = (uint8_t)b;
            special |= (__ballot(b >= 253u) != 0ull ? 1u : 0u) << j;
        }
        if ((tid & 63u) == 0u) {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                s_special[(tid >> 6) * 8 + j] = (uint8_t)((special >> j) & 1u);
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
        const uint32_t *s_in = reinterpret_cast<const uint32_t *>(s_out) + rg * 32u * 32u + cg;
#pragma unroll
        for (int i = 0; i < 32; ++i)
            w[i] = s_in[i * 32];
        __syncthreads(); // every slice is in registers before the tile buffer takes the results
    }

    // ---- the lane's view: its k-block kb, its 128-row group g
    const uint32_t kb = cg >> 2, g = rg >> 2;
    const bool special = (s_special[(2 * g) * 8 + kb] | s_special[(2 * g + 1) * 8 + kb]) != 0u;
    const uint8_t *my_row_sf = &s_row_sf[kb * TILE_M + rg * 32u];
    uint32_t sb[8]; // the 32 row-scale bytes of this slice: byte i%4 of dword i/4 is row i
    {
        const u32x4 s0 = reinterpret_cast<const u32x4 *>(my_row_sf)[0];
        const u32x4 s1 = reinterpret_cast<const u32x4 *>(my_row_sf)[1];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            sb[q] = s0[q];
            sb[4 + q] = s1[q];
        }
    }

    // ---- pass 1: column maxima of |value| over the lane's 32 rows (rows that do not exist are zeros)
    float amax[8];
#pragma unroll
    for (int c = 0; c < 8; ++c)
        amax[c] = 0.0f;
    if (active && !special) {
        static_for<16>([&](auto ip) {
            constexpr int i = 2 * decltype(ip)::value;
            const float sa = row_scale_operand<i>(sb), sbb = row_scale_operand<i + 1>(sb);
            static_for<4>([&](auto jp) {
                constexpr int j = decltype(jp)::value;
                const f32x2 fa = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[i], sa, j);
                const f32x2 fb = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[i + 1], sbb, j);
                amax[2 * j] = max3_abs_nan(fa.x, fb.x, amax[2 * j]);
                amax[2 * j + 1] = max3_abs_nan(fa.y, fb.y, amax[2 * j + 1]);
            });
        });
    }
    if (in_cols) {
        u32x4 *dst = reinterpret_cast<u32x4 *>(&s_amax[rg * TILE_K + cg * 8u]);
        dst[0] = u32x4{f2u(amax[0]), f2u(amax[1]), f2u(amax[2]), f2u(amax[3])};
        dst[1] = u32x4{f2u(amax[4]), f2u(amax[5]), f2u(amax[6]), f2u(amax[7])};
    }
    __syncthreads();

    // ---- the group's column maxima -> Emax -> the encoder's operand exponent Emax - 9
    float enc[8];
    bool slow = special;
    if (active) {
        uint32_t mx[8];
#pragma unroll
        for (int c = 0; c < 8; ++c)
            mx[c] = 0u;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const u32x4 *src = reinterpret_cast<const u32x4 *>(&s_amax[(4u * g + i) * TILE_K + cg * 8u]);
            const u32x4 p0 = src[0], p1 = src[1];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                mx[c] = max(mx[c], p0[c]); // non-negative floats order like their bit patterns
                mx[4 + c] = max(mx[4 + c], p1[c]);
            }
        }
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const uint32_t ef = mx[c] >> 23;
            slow |= mx[c] != 0u && ef < 8u;               // a maximum below 2^-118: operand exponent negative
            enc[c] = u2f((mx[c] != 0u ? ef - 8u : 127u) << 23);
        }
    }

    // ---- group scales: k-row t of the tile, one float per 128-row group
    if (tid < cols) {
        const uint32_t kbt = tid >> 5;
        uint32_t bits[2];
#pragma unroll
        for (int gg = 0; gg < 2; ++gg) {
            if ((s_special[(2 * gg) * 8 + kbt] | s_special[(2 * gg + 1) * 8 + kbt]) == 0u) {
                uint32_t m = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    m = max(m, f2u(s_amax[(4 * gg + i) * TILE_K + tid]));
                bits[gg] = scale_bits_of_emax(emax_of_amax_bits(m), m != 0u);
            } else if ((uint32_t)gg < n_g) {
                const int emax = group_emax_int(tile_src, pitch, &s_row_sf[kbt * TILE_M], tid, gg * 128u,
                                                min(128u, n_rows - gg * 128u));
                bits[gg] = emax >= GROUP_HAS_NAN - 1 ? 0x7FC00000u : scale_bits_of_emax(emax, emax >= 0);
            } else {
                bits[gg] = 0u;
            }
        }
        float *dst = out_s + (size_t)(k0 + tid) * pitch_s + m0 / 128u;
        // one request per k-row: an expert's scale rows start at any multiple of 4 bytes
        if (n_g == 2u)
            *reinterpret_cast<u64_unaligned *>(dst) = ((uint64_t)bits[1] << 32) | bits[0];
        else if (n_g == 1u)
            dst[0] = u2f(bits[0]);
    }

    // ---- pass 2: decode again, re-quantize pairs of rows into output bytes
    const uint32_t slot0 = (2u * rg + cg) & 15u; // 16-byte slots of rows 0..15 / 16..31 of the slice
    const uint32_t slot1 = (2u * rg + 1u + cg) & 15u;
    if (active && !slow) {
        static_for<4>([&](auto jp) {
            constexpr int j = decltype(jp)::value; // nibble byte: columns 2j, 2j+1
            uint32_t o[2][8];
            static_for<8>([&](auto rp) {
                constexpr int r = decltype(rp)::value; // rows 4r..4r+3 -> dword r of both columns
                const f32x2 f0 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[4 * r], row_scale_operand<4 * r>(sb), j);
                const f32x2 f1 =
                    __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[4 * r + 1], row_scale_operand<4 * r + 1>(sb), j);
                const f32x2 f2 =
                    __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[4 * r + 2], row_scale_operand<4 * r + 2>(sb), j);
                const f32x2 f3 =
                    __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[4 * r + 3], row_scale_operand<4 * r + 3>(sb), j);
                s16x2 e0, e1; // no initial value needed: both words are written
                asm volatile("" : "=v"(e0), "=v"(e1));
                e0 = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(e0, f0.x, f1.x, enc[2 * j], false);
                e0 = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(e0, f2.x, f3.x, enc[2 * j], true);
                e1 = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(e1, f0.y, f1.y, enc[2 * j + 1], false);
                e1 = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(e1, f2.y, f3.y, enc[2 * j + 1], true);
                o[0][r] = __builtin_bit_cast(uint32_t, e0);
                o[1][r] = __builtin_bit_cast(uint32_t, e1);
            });
#pragma unroll
            for (int cc = 0; cc < 2; ++cc) {
                const uint32_t row = (2 * j + cc) * 32u + cg; // LDS k-row of column 2j+cc
                s_out[row * 16u + slot0] = u32x4{o[cc][0], o[cc][1], o[cc][2], o[cc][3]};
                s_out[row * 16u + slot1] = u32x4{o[cc][4], o[cc][5], o[cc][6], o[cc][7]};
            }
        });
    } else if (active) {
        // the integer path: per column the group's Emax from all of its rows, then this lane's 32
        // elements (nibbles read again from global memory) byte by byte into its own LDS slots
        uint8_t *bytes = reinterpret_cast<uint8_t *>(s_out);
        const uint32_t r0 = g * 128u, n = min(128u, n_rows - r0);
#pragma nounroll
        for (uint32_t c = 0; c < 8u; ++c) {
            int emax = group_emax_int(tile_src, pitch, &s_row_sf[kb * TILE_M], cg * 8u + c, r0, n);
            emax = emax >= GROUP_HAS_NAN - 1 ? emax - GROUP_HAS_NAN : emax;
#pragma nounroll
            for (uint32_t i = 0; i < 32u && rg * 32u + i < n_rows; ++i) {
                const uint32_t b = my_row_sf[i];
                const uint32_t byte = tile_src[(size_t)(rg * 32u + i) * pitch + cg * 4u + (c >> 1)];
                const uint32_t nib = ((c & 1u) ? byte >> 4 : byte) & 0xFu;
                const uint32_t out = b == 255u ? 0x7Fu : e4m3_requant_int(nib, b, emax);
                bytes[((c * 32u + cg) * 16u + (i < 16u ? slot0 : slot1)) * 16u + (i & 15u)] = (uint8_t)out;
            }
        }
    }
    __syncthreads();

    write_tile_out(s_out, out_x + (size_t)k0 * pitch_x + m0, out_x, pitch_x, cols, n_rows, tid);
}

hipError_t launch_row_to_fp8_col_requant(const uint8_t *q_row, const uint8_t *sf_row, const int32_t *expert_offsets,
                                         int32_t num_experts, int64_t M, int64_t K, uint8_t *x_col,
                                         float *x_col_scale, hipStream_t stream)
{
    fp8col_requant::Args a;
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
    hipLaunchKernelGGL(row_to_fp8_col_requant_kernel, grid, dim3(T_THREADS), 0, stream, a);
    return hipGetLastError();
}

} // namespace mxfp4
