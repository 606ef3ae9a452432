// Row-blocked MXFP4 -> column-blocked MXFP4 (stored transposed), gfx950.
//
// Paper sec. 3.4: de-quantization, transposition and re-quantization fused into one pass
// through on-chip memory, so the matrix is read once and written once.  Every element
// takes its exact value e2m1 * 2^(b_row - 127); each 32x1 run along m is re-quantized with
// the scale rule and rounding of sec. 3.1.
//
// Work split.  A workgroup of 256 lanes owns a 256 (m) x 256 (k) tile, the unit that makes
// both global reads and global writes 128-byte contiguous (512-row tiles with 512 lanes
// were measured too: fewer scale requests, but slower overall).  Inside, the unit of work is the
// 32x32 block of the method: lane (rg, cg) owns rows 32*rg..32*rg+31 and the 8 columns
// 8*cg..8*cg+7, i.e. one 32x8 slice of a 32x32 block, as 32 dwords of nibbles (one per row).
//   pass 1: v_cvt_scalef32_pk_f32_fp4 (row scale applied by the instruction, two columns
//           per issue) and a running |max| per column -> 8 column maxima -> 8 UE8M0 bytes
//           by exponent-field arithmetic.
//   pass 2: the same decode again (cheaper than keeping 256 floats live), then
//           v_cvt_scalef32_pk_fp4_f32 takes the values of rows (m, m+1) of one column and
//           emits the output byte directly: the register pairing IS the transposition of
//           the 32x32 block, no nibble shuffling is needed.
// The 8 x 16 B per lane then go through an LDS tile (swizzled so that both the 16-byte
// writes and the linear read-back are bank-conflict free) to leave as full 128-byte rows.
// Workgroups take their tiles in an XCD-aware order (tile_of_workgroup), which is what keeps
// the HBM traffic at the algorithmic 0.53125 B read + 0.53125 B written per element.
#include "mxfp4_device.hpp"
#include "mxfp4_kernels.hpp"

namespace mxfp4 {

constexpr int NRG = 8;              // 32-row groups per tile
constexpr int T_THREADS = 32 * NRG; // one lane per (row group, 8-column group)
constexpr int TILE_M = 32 * NRG;
constexpr int TILE_K = 256;
// row scales of one k-block in LDS; the pad spreads the k-blocks over the banks
constexpr int SF_STRIDE = TILE_M + 16;

struct RowToColArgs {
    const uint8_t *q_row;
    const uint8_t *sf_row;
    uint8_t *q_col;
    uint8_t *sf_col;
    const int32_t *expert_offsets; // nullptr: one group of M rows
    int32_t num_experts;
    uint32_t M; // total rows
    uint32_t K;
    uint32_t tiles_m; // 256-row tiles (an upper bound when grouped)
    uint32_t tiles_k; // 256-column tiles
    uint32_t stage_in; // full tiles fetch their nibbles with 16-byte loads and re-slice them through LDS
    uint32_t mbm;      // row tiles per macro block of the tile order (one matrix; experts: see the lookup)
};

// Macro block of the tile order: 4 column tiles; row tiles by macro_block_rows for one matrix (32 at
// [65536,7168], where over rotated buffers 8 / 16 / 64 row tiles took 103 / 108 / 98 us against 93 and 1, 2, 7, 14
// or 28 column tiles made no difference), at most MBM_MAX inside an expert of a grouped launch.
constexpr uint32_t MBM_MAX = 64, MBK = 4;

// The nibbles are read once: non-temporal loads.
__device__ __forceinline__ uint32_t load_nibbles(const uint32_t *p)
{
    return __builtin_nontemporal_load(p);
}

// One lane's 32x8 slice through the hardware conversions, in two steps with the column scales between them
// (the workgroup sends the scale bytes off before it re-quantizes).  Exact while every value
// e2m1 * 2^(b-127) is an FP32 number, i.e. for row-scale bytes up to 252
// (6 * 2^125 < 2^128; the smallest, 0.5 * 2^-127, is an FP32 subnormal).
// Step 1: the UE8M0 bytes of the slice's 8 columns.
__device__ __forceinline__ void column_scales_hw(const uint32_t (&w)[32], const uint32_t (&sb)[8], uint32_t (&cb)[8])
{
    // column maxima of |value| (no NaN can occur: NaN row scales never get here)
    float amax[8];
#pragma unroll
    for (int c = 0; c < 8; ++c)
        amax[c] = 0.0f;
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
    // the sec. 3.1 rule on the exponent field.  A maximum with at most two significant bits (1.0 or 1.5
    // times a power of two) never exceeds 1.5 * 2^e, so the byte is its exponent field minus 2, clamped
    // at 0; zero and FP32 subnormals give 0.
#pragma unroll
    for (int c = 0; c < 8; ++c)
        cb[c] = max(f2u(amax[c]) >> 23, 2u) - 2u;
}

// Step 2: decode again (cheaper than keeping 256 floats live) and re-quantize pairs of rows into output
// bytes: v_cvt_scalef32_pk_fp4_f32 takes rows (m, m+1) of one column.
__device__ __forceinline__ void requant_rows_hw(uint32_t (&w)[32], uint32_t (&sb)[8], const uint32_t (&cb)[8],
                                                uint32_t (&o)[8][4])
{
    float cs[8];
#pragma unroll
    for (int c = 0; c < 8; ++c)
        cs[c] = u2f(cb[c] << 23);
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
        for (int g = 0; g < 4; ++g)
            asm volatile("" : "=v"(o[c][g])); // no initial value needed: all four bytes are written
    static_for<16>([&](auto ip) {
        constexpr int i = 2 * decltype(ip)::value;
        constexpr int g = i >> 3, sel = (i >> 1) & 3; // output dword and byte of rows (i, i+1)
        const float sa = row_scale_operand<i>(sb), sbb = row_scale_operand<i + 1>(sb);
        static_for<4>([&](auto jp) {
            constexpr int j = decltype(jp)::value;
            const f32x2 fa = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[i], sa, j);
            const f32x2 fb = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w[i + 1], sbb, j);
            o[2 * j][g] = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(o[2 * j][g], fa.x, fb.x, cs[2 * j], sel);
            o[2 * j + 1][g] =
                __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(o[2 * j + 1][g], fa.y, fb.y, cs[2 * j + 1], sel);
        });
    });
}

// The same slice in integers, for row-scale bytes 253 and 254, whose largest values
// (4 and 6 times 2^126 or 2^127) exceed FP32.  Never taken by real activations, so it is
// written for size, not speed: rolled loops that re-read the nibbles (they are still in
// cache) and the staged row scales, and write straight into the LDS output tile.
// Every non-zero E2M1 value is (1 + M/2) * 2^(E-1) with the pair (E, M) = (field, mantissa),
// except the subnormal 0.5 = 1.0 * 2^-1, i.e. (0, 0).  With at most two significant bits,
// ceil(log2(x/6)) = floor(log2 x) - 2, so the column byte is max(0, max(b_row + E) - 3).
// Relative to it, t = 2*(b_row + E - b_col) + M orders the values; t >= 2 are E2M1 normals
// and stay exact (code t), and below that RTNE gives t = 1 -> 1.0 (tie .75, even code 2),
// t = 0 and -1 -> 0.5 (code 1), t = -2 -> 0 (tie .25), lower -> 0.
// Only the first n_valid rows of the slice exist (fewer than 32 at the ragged end of a split).
__device__ __noinline__ uint64_t requant_slice_int(const uint8_t *src, size_t src_pitch, const uint8_t *row_sf,
                                                   uint32_t *out_row0, uint32_t out_row_stride, int n_valid)
{
    uint64_t col_bytes = 0;
#pragma nounroll
    for (int c = 0; c < 8; ++c) {
        int emax = -1024;
#pragma nounroll
        for (int i = 0; i < n_valid; ++i) {
            const uint32_t wi = *reinterpret_cast<const uint32_t *>(src + (size_t)i * src_pitch);
            const int mag = (int)(wi >> (4 * c)) & 7;
            if (mag)
                emax = max(emax, (int)row_sf[i] + (mag >> 1));
        }
        const int bc = max(0, emax - 3);
        col_bytes |= (uint64_t)bc << (8 * c);
#pragma nounroll
        for (int g = 0; g < 4; ++g) {
            uint32_t acc = 0;
#pragma nounroll
            for (int i8 = 0; i8 < 8; ++i8) {
                const int i = g * 8 + i8;
                if (i >= n_valid)
                    break; // the nibbles of rows that do not exist stay 0
                const uint32_t wi = *reinterpret_cast<const uint32_t *>(src + (size_t)i * src_pitch);
                const uint32_t nib = (wi >> (4 * c)) & 0xFu;
                const int mag = (int)(nib & 7u);
                const int em = mag == 1 ? 0 : mag; // 2*E + M of the normalised value
                const int t2 = max(em + 2 * ((int)row_sf[i] - bc) + 2, 0);
                int code = min(7, max(t2 - 2, (t2 + 1) >> 1));
                code = mag ? code : 0;
                acc |= ((nib & 8u) | (uint32_t)code) << (4 * i8);
            }
            out_row0[c * out_row_stride + g] = acc;
        }
    }
    return col_bytes;
}

// One tile per workgroup and two barriers (three when the nibbles are re-sliced through LDS): the column
// scales get their own 2 KiB of LDS, so that after the conversion the scale bytes and the nibbles leave without
// further synchronisation.  The scale bytes sit in LDS so that no access piles up on one bank: the k-blocks of the
// row scales are SF_STRIDE = 272 bytes apart (the eight 32-byte reads of a wave fall on different banks), and the
// byte of column cg*8 + c goes to slot c*32 + cg, which lane tid reads back linearly (with slot k = cg*8 + c the
// eight byte writes of a lane met 16-way conflicts, 70 % of the kernel's LDS cycles).
//
// What bounds it, measured at [65536,7168] over three rotated buffer sets, so that every byte comes from and
// goes to HBM and not the 256 MB memory-side cache (93 us = 5.4 TB/s as built; all forms below bit-identical to
// it unless they leave something out):
//  * A kernel that only moves the nibbles in this access pattern (the same 16-byte loads of 256 x 128-byte rows,
//    one barrier, the same 256 transposed 128-byte k-rows out, no LDS tile, no arithmetic, no scales): 79 us.
//    This kernel without its scale traffic: 83 us; with both scale planes in a layout where a tile's 2 KiB are
//    contiguous: 86 us.  So the scale planes, 6 % of the bytes, cost 10 us as they are laid out (8 bytes per row
//    and per k-row: 40 % of the requests to the L2), 3 us would be their share.  Without the column-scale
//    stores 88 us, without the row-scale loads 90 us.  Merging the pieces of four tiles into one 32-byte request
//    gained 3.7 us on the loads and nothing on the stores; row scales through scalar loads (one 8-byte
//    s_load per row, dealt to the lanes with v_writelane): 94-97 us.  Workgroups of 512 lanes that take two
//    tiles next to each other along k, each half in its own LDS as here, with one 16-byte request for the row
//    scales of both: 98 us against 90 (the bare mover with the scale traffic gains 3 us from that request
//    shape; two 74 KB workgroups per CU and barriers over eight waves lose more).
//  * Plain instead of non-temporal stores for the k-rows: 104 us (they only pay when the output is rewritten
//    in place and stays in the cache: 89 against 93 us); write-through (sc1, sc0 sc1): 103 us; non-temporal
//    column-scale stores: 142 us; non-temporal row-scale loads: 128 us.
//  * Workgroups that stay resident and take one tile after the other lose 10 % whatever they do between the
//    tiles, the bare copy included (79 -> 87 us with 4 per CU, by a fixed stride or by claiming tile numbers from
//    a counter in global memory); this kernel in that form 104-110 us, also with a fifth wave that does nothing
//    but move finished tiles from LDS to memory so that the converting waves never wait for a store.  The
//    hardware's own dispatch of one short workgroup per tile is the better scheduler here.
//  * Macro blocks of 8 / 16 / 64 row tiles: 103 / 108 / 98 us; 1 to 28 column tiles: no difference.  Dword loads
//    (one per row and lane) instead of the 16-byte loads re-sliced through LDS: 95 us.
__global__ void __launch_bounds__(T_THREADS) row_to_col_kernel(const RowToColArgs a)
{
    __shared__ u32x4 s_out[TILE_K * NRG];                // [c*32 + cg][slot]: 256 k-rows x 128 B
    __shared__ alignas(16) uint8_t s_row_sf[8 * SF_STRIDE]; // [k-block of the tile][row]
    __shared__ alignas(16) uint8_t s_col_sf[TILE_K * NRG]; // [slot c*32 + cg of column cg*8 + c][row group]
    __shared__ uint8_t s_special[NRG];                   // per row group: bit kb set = a scale byte >= 253

    // ---- which tile, and which rows: the whole matrix, or one expert's slice of any length (uniform
    // per workgroup)
    uint32_t strip, tile_k;
    uint32_t row_base = 0, rows = a.M, bytes_before = 0, blocks_before = 0;
    if (a.expert_offsets) {
        if (!tile_of_grouped_workgroup<TILE_M, 2, 32, MBM_MAX, MBK>(a.expert_offsets, a.num_experts, blockIdx.x, a.tiles_k,
                                                                &strip, &tile_k, &row_base, &rows, &bytes_before,
                                                                &blocks_before))
            return;
    } else if (!tile_of_workgroup<MBK>(blockIdx.x, a.tiles_m, a.tiles_k, a.mbm, &strip, &tile_k)) {
        return;
    }
    const uint32_t m0 = strip * TILE_M;
    if (m0 >= rows)
        return;
    const uint32_t n_rows = min((uint32_t)TILE_M, rows - m0); // rows present: 1..256
    const uint32_t n_rg = (n_rows + 31u) / 32u;               // row groups present, the last maybe partial
    const uint32_t k0 = tile_k * TILE_K;
    const uint32_t cols = min((uint32_t)TILE_K, a.K - k0); // 128 or 256
    const uint32_t Kb = a.K / 32u;

    // expert e's output is its own dense [K, ceil(rows/2)] and [K, ceil(rows/32)], after those of
    // the experts before it
    uint8_t *out_q = a.q_col + (size_t)a.K * bytes_before;
    uint8_t *out_sf = a.sf_col + (size_t)a.K * blocks_before;
    const size_t pitch_q = (rows + 1u) / 2u, pitch_sf = (rows + 31u) / 32u;

    const uint32_t tid = threadIdx.x;
    const uint32_t rg = tid >> 5, cg = tid & 31u;
    const uint32_t pitch = a.K / 2u;
    // results go to LDS row (c*32 + cg), 16-byte slot rotated by the column group, so that
    // consecutive lanes write different banks and the read-back is linear
    const uint32_t slot = (rg + (cg >> 1)) & (NRG - 1u);
    const uint32_t lane_off = rg * 32u * pitch + cg * 4u;
    const bool active = rg * 32u < n_rows && cg * 8u < cols;

    // the tile's row scales: thread t takes row t, one 8-byte request (4 bytes for a 128-column tile)
    uint32_t lo = 0, hi = 0;
    auto load_sf = [&]() {
        if (tid < n_rows) {
            const uint8_t *p = a.sf_row + (size_t)(row_base + m0 + tid) * Kb + k0 / 32u;
            if (cols > 128u) { // one request at any 4-byte alignment
                const u32x2 v = *reinterpret_cast<const u32x2_unaligned *>(p);
                lo = v.x;
                hi = v.y;
            } else {
                lo = reinterpret_cast<const uint32_t *>(p)[0];
                hi = 0u;
            }
        }
    };
    // the 32x8 slice of a lane: one dword (8 nibbles) per row, from a uniform row pointer plus a
    // 32-bit lane offset (one address register, not 32 pairs)
    uint32_t w[32];
    auto load_slice = [&]() {
        if (active) {
            const uint8_t *tile_src = a.q_row + (size_t)(row_base + m0) * pitch + k0 / 2u;
            if (n_rows == (uint32_t)TILE_M) {
#pragma unroll
                for (int i = 0; i < 32; ++i)
                    w[i] = load_nibbles(reinterpret_cast<const uint32_t *>(tile_src + (size_t)i * pitch + lane_off));
            } else {
                // ragged end of a split: rows past it count as zeros (read from the last row, then cleared)
                const uint32_t last = n_rows - 1u - rg * 32u;
#pragma unroll
                for (int i = 0; i < 32; ++i) {
                    const uint32_t v =
                        load_nibbles(reinterpret_cast<const uint32_t *>(tile_src + lane_off + min((uint32_t)i, last) * pitch));
                    w[i] = (uint32_t)i <= last ? v : 0u;
                }
            }
        }
    };
    // With many tiles per CU a full tile arrives through 16-byte loads (8 rows x 128 bytes per wave
    // instruction instead of 2) and is cut into the lanes' 32 x 8 slices through the tile buffer: a wave
    // fetches the 64 rows of its own two row groups, row-major.  At [65536,7168] 93 us against 95.  Over rotated
    // buffers the dword loads win up to 640 tiles by 1-3 % ([16384,2048] 9.3 against 9.7 us), at 768 tiles the two
    // are equal, from 896 on ([8192,7168], [32768,2048], [16384,4096]) the 16-byte loads win by 6-8 %: the launcher
    // asks for them from three tiles per compute unit on.
    const bool staged = a.stage_in != 0u && n_rows == (uint32_t)TILE_M && cols == (uint32_t)TILE_K &&
                        (reinterpret_cast<uintptr_t>(a.q_row) & 15u) == 0u;
    u32x4 stage_v[8];
    if (staged) {
        const uint32_t wv = tid >> 6, lane = tid & 63u;
        const uint8_t *src = a.q_row + (size_t)(row_base + m0) * pitch + k0 / 2u +
                             (size_t)(wv * 64u + (lane >> 3)) * pitch + (lane & 7u) * 16u;
#pragma unroll
        for (int j = 0; j < 8; ++j)
            stage_v[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + (size_t)(j * 8) * pitch));
    } else {
        load_slice();
    }
    load_sf();
    // ---- stage the row scales.  A wave stages two row groups; one ballot per k-block tells which
    // (row group, k-block) pairs hold a byte of 253 or more (beyond FP32, or NaN).
    {
        if (tid < TILE_M) { // rows that do not exist are staged as byte 0
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                s_row_sf[j * SF_STRIDE + tid] = (uint8_t)(lo >> (8 * j));
                s_row_sf[(4 + j) * SF_STRIDE + tid] = (uint8_t)(hi >> (8 * j));
            }
        }
        // a byte is 253 or more when its top bit is set and its low seven bits plus 3 reach 128: one test
        // for the 8 bytes of a row and one ballot for the wave; the per-k-block ballots only run when it fires
        uint32_t special_lo = 0, special_hi = 0;
        const uint32_t big = ((((lo & 0x7F7F7F7Fu) + 0x03030303u) & lo) | (((hi & 0x7F7F7F7Fu) + 0x03030303u) & hi)) &
                             0x80808080u;
        if (__ballot(big != 0u) != 0ull) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t b = ((j < 4 ? lo : hi) >> (8 * (j & 3))) & 0xFFu;
                const uint64_t m = __ballot(b >= 253u);
                special_lo |= ((uint32_t)m != 0u ? 1u : 0u) << j;
                special_hi |= ((uint32_t)(m >> 32) != 0u ? 1u : 0u) << j;
            }
        }
        if ((tid & 63u) == 0u) {
            s_special[(tid >> 6) * 2] = (uint8_t)special_lo;
            s_special[(tid >> 6) * 2 + 1] = (uint8_t)special_hi;
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

    // ---- step 1: the column scales of every slice, and the slices that take the integer path in full
    uint32_t sb[8], cb[8];
    bool hw = false; // this lane's slice goes through the hardware conversions
    if (active) {
        const uint8_t *my_row_sf = &s_row_sf[(cg >> 2) * SF_STRIDE + rg * 32u];
        uint64_t col_bytes;
        if (((s_special[rg] >> (cg >> 2)) & 1u) == 0u) {
            hw = true;
            const u32x4 s0 = reinterpret_cast<const u32x4 *>(my_row_sf)[0];
            const u32x4 s1 = reinterpret_cast<const u32x4 *>(my_row_sf)[1];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                sb[g] = s0[g];
                sb[4 + g] = s1[g];
            }
            column_scales_hw(w, sb, cb);
            uint32_t cb_lo = 0, cb_hi = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                cb_lo |= cb[c] << (8 * c);
                cb_hi |= cb[4 + c] << (8 * c);
            }
            col_bytes = ((uint64_t)cb_hi << 32) | cb_lo;
        } else {
            bool poisoned = false; // a NaN row scale touches all 8 columns of the slice
            for (int i = 0; i < 32; ++i)
                poisoned |= my_row_sf[i] == 255u;
            if (poisoned) {
#pragma unroll
                for (int c = 0; c < 8; ++c)
                    s_out[(c * 32 + cg) * NRG + slot] = u32x4{0u, 0u, 0u, 0u};
                col_bytes = ~(uint64_t)0;
            } else {
                const uint8_t *tile_src = a.q_row + (size_t)(row_base + m0) * pitch + k0 / 2u;
                col_bytes = requant_slice_int(tile_src + lane_off, pitch, my_row_sf,
                                              reinterpret_cast<uint32_t *>(&s_out[cg * NRG + slot]), 32 * NRG * 4,
                                              (int)min(32u, n_rows - rg * 32u));
            }
        }
#pragma unroll
        for (int c = 0; c < 8; ++c)
            s_col_sf[(c * 32 + cg) * NRG + rg] = (uint8_t)(col_bytes >> (8 * c));
    }
    __syncthreads();

    // ---- the column scales leave now, one request per k-row, while the nibbles are still being re-quantized
    // (93.1 -> 90.8 us at [65536,7168] against sending them off together with the nibbles at the end).
    const uint32_t sf_k = (tid & 31u) * 8u + (tid >> 5); // slot tid of the staged column scales is column sf_k
    if (sf_k < cols) {
        uint8_t *dst = out_sf + (size_t)(k0 + sf_k) * pitch_sf + m0 / 32u;
        const u32x2 v = *reinterpret_cast<const u32x2 *>(&s_col_sf[tid * NRG]);
        // one request per k-row at any alignment (the pitch of an expert's scale rows is any number of
        // bytes): 8 bytes for a full tile, the pieces of store_head_bytes for a tile that ends early
        if (n_rg == 8u)
            *reinterpret_cast<u64_unaligned *>(dst) = ((uint64_t)v.y << 32) | v.x;
        else
            store_head_bytes(dst, u32x4{v.x, v.y, 0u, 0u}, n_rg);
    }

    // ---- step 2: re-quantize into the tile buffer
    if (hw) {
        uint32_t o[8][4];
        requant_rows_hw(w, sb, cb, o);
#pragma unroll
        for (int c = 0; c < 8; ++c)
            s_out[(c * 32 + cg) * NRG + slot] = u32x4{o[c][0], o[c][1], o[c][2], o[c][3]};
    }
    __syncthreads();

    // ---- out: the nibbles, 8 lanes per k-row with 128 contiguous bytes each.  Chunk u*256 + tid of the LDS
    // tile is row (u*32 + tid/8), slot tid%8: column k = (tid/8)*8 + u.
    {
        const uint32_t cgx = tid / NRG;
        const uint32_t part = ((tid & (NRG - 1u)) - (cgx >> 1)) & (NRG - 1u);
        uint8_t *dst = out_q + (size_t)(k0 + cgx * 8u) * pitch_q + m0 / 2u + part * 16u;
        // bytes of this lane's 16 (= 32 rows) that exist: fewer at the ragged end of a split, where
        // k-rows also start at any byte (global memory takes unaligned vector stores)
        const uint32_t have = part * 32u < n_rows ? min(16u, (n_rows - part * 32u + 1u) / 2u) : 0u;
        // Non-temporal stores where a tile's 128-byte piece of a k-row consists of whole 64-byte segments (over
        // rotated buffers at [65536,7168]: 93 us against 104 with plain stores).  Where the pitch of a split
        // puts the pieces across segment boundaries the halves of a segment come from two workgroups and have to
        // meet in the L2 first: plain stores (32 splits of 1984 rows, pitch 992 bytes: 2.7 ns per row
        // non-temporal, 1.7 plain).
        const bool segments64 = ((reinterpret_cast<uintptr_t>(out_q) | pitch_q) & 63u) == 0u;
        if (cgx * 8u < cols && have != 0u) {
            if (have == 16u && segments64) {
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    __builtin_nontemporal_store(s_out[u * T_THREADS + tid], reinterpret_cast<u32x4 *>(dst + (size_t)u * pitch_q));
            } else if (have == 16u) {
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    *reinterpret_cast<u32x4_unaligned *>(dst + (size_t)u * pitch_q) = s_out[u * T_THREADS + tid];
            } else {
#pragma nounroll
                for (int u = 0; u < 8; ++u)
                    store_head_bytes(dst + (size_t)u * pitch_q, s_out[u * T_THREADS + tid], have);
            }
        }
    }
}

hipError_t launch_row_to_col(const uint8_t *q_row, const uint8_t *sf_row, const int32_t *expert_offsets,
                             int32_t num_experts, int64_t M, int64_t K, uint8_t *q_col, uint8_t *sf_col,
                             hipStream_t stream)
{
    RowToColArgs a;
    a.q_row = q_row;
    a.sf_row = sf_row;
    a.q_col = q_col;
    a.sf_col = sf_col;
    a.expert_offsets = expert_offsets;
    a.num_experts = num_experts;
    a.M = (uint32_t)M;
    a.K = (uint32_t)K;
    // upper bound on the number of row tiles: every expert may end in a partial one
    a.tiles_m = (uint32_t)((M + TILE_M - 1) / TILE_M + (expert_offsets ? num_experts : 0));
    a.tiles_k = (uint32_t)((K + TILE_K - 1) / TILE_K);
    a.mbm = macro_block_rows(a.tiles_m);
    const uint32_t total = a.tiles_m * a.tiles_k;
    a.stage_in = total >= 3u * compute_units() ? 1u : 0u; // at least 3 tiles per compute unit
    const dim3 grid((total + NUM_XCD - 1) / NUM_XCD * NUM_XCD);
    hipLaunchKernelGGL(row_to_col_kernel, grid, dim3(T_THREADS), 0, stream, a);
    return hipGetLastError();
}

} // namespace mxfp4
