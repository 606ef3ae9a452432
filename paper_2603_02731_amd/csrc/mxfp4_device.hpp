// Device-side helpers shared by the gfx950 conversion kernels.
//
// Hardware facts the kernels rely on (each checked exhaustively by the GPU parity tests):
//  * v_cvt_pk_f32_fp8 decodes OCP E4M3 exactly, subnormals and NaN included.
//  * v_cvt_scalef32_pk_fp4_f32 computes RTNE(src / 2^(E-127)) onto E2M1 with gradual
//    underflow and saturation, E being bits 30:23 of the scale operand (sign and mantissa
//    of the scale are ignored, E = 0 means 2^-127), keeps the sign of zero results, and
//    honours FP32 subnormal sources.
//  * v_cvt_scalef32_pk_f32_fp4 returns e2m1 * 2^(E-127) exactly, as FP32 subnormals where
//    needed.
//  * v_cvt_scalef32_pk_fp8_f32 computes RTNE(src / 2^(E-127)) onto OCP E4M3 with gradual
//    underflow, keeps the sign of zero results, and puts its first source in the low byte.
//  * v_maximum3_f32 propagates NaN.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

namespace mxfp4 {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
// The same through pointers of any alignment (global memory takes unaligned vector accesses).
typedef u32x4 __attribute__((aligned(1))) u32x4_unaligned;
typedef u32x2 __attribute__((aligned(1))) u32x2_unaligned;
typedef uint64_t __attribute__((aligned(1))) u64_unaligned;
typedef uint32_t __attribute__((aligned(1))) u32_unaligned;
typedef uint16_t __attribute__((aligned(1))) u16_unaligned;

__device__ __forceinline__ uint32_t f2u(float f) { return __builtin_bit_cast(uint32_t, f); }
__device__ __forceinline__ float u2f(uint32_t u) { return __builtin_bit_cast(float, u); }

// Byte permute: the result's byte i is byte sel[i] of the 8-byte pool {hi:lo}
// (selector values 0..3 pick from lo, 4..7 from hi).
__device__ __forceinline__ uint32_t perm(uint32_t hi, uint32_t lo, uint32_t sel)
{
    return __builtin_amdgcn_perm(hi, lo, sel);
}

// Value of another lane of the same row of 16, selected by a DPP control.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_read(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
constexpr int DPP_QUAD_XOR1 = 0xB1; // quad_perm [1,0,3,2]
constexpr int DPP_QUAD_XOR2 = 0x4E; // quad_perm [2,3,0,1]
constexpr int DPP_ROW_HALF_MIRROR = 0x141; // lane i <-> lane 7-i inside each group of 8
constexpr int DPP_ROW_MIRROR = 0x140;      // lane i <-> lane 15-i inside each row of 16

// Value of lane i+4 of the same row of 16 lanes (0 where there is none), by DPP.
__device__ __forceinline__ uint32_t row_shift_left4(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x104 /* row_shl:4 */, 0xF, 0xF, true);
}

// Value of lane i+8 of the same row of 16 lanes (0 where there is none), by DPP.
__device__ __forceinline__ uint32_t row_shift_left8(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x108 /* row_shl:8 */, 0xF, 0xF, true);
}

// NaN-propagating maximum of |a|, |b| and c.
__device__ __forceinline__ float max3_abs_nan(float a, float b, float c)
{
    return __builtin_elementwise_maximum(
        __builtin_elementwise_maximum(__builtin_fabsf(a), __builtin_fabsf(b)), c);
}

// UE8M0 byte of the block scale for a block maximum given as FP32 bits (sign clear):
// the smallest k with gmax <= 6 * 2^k, biased by 127 and clamped to [0,254]
// (paper sec. 3.1, evaluated on the exponent field as in sec. 3.4).
// gmax = 1.f * 2^(e-127): gmax <= 6 * 2^k = 1.5 * 2^(k+2)  <=>  k = e-127-2 when f <= 1.5,
// one more otherwise.  Zero and FP32 subnormals land on byte 0 through the clamp,
// +inf gives 254, NaN gives 0xFF.
__device__ __forceinline__ uint32_t ue8m0_of_block_max(uint32_t gmax_bits)
{
    int e = (int)(gmax_bits >> 23);
    uint32_t mant = gmax_bits & 0x7FFFFFu;
    int b = e - 2 + (mant > 0x400000u ? 1 : 0);
    b = b < 0 ? 0 : b;
    b = gmax_bits == 0x7F800000u ? 254 : b;
    b = gmax_bits > 0x7F800000u ? 255 : b;
    return (uint32_t)b;
}

// Scale operand of row I of a 32-row slice whose UE8M0 bytes are packed four to a dword (byte
// I%4 of dword I/4): the byte moved into bits 30:23 with one shift.  What lands in the sign and
// mantissa bits belongs to the neighbouring bytes; the conversion instructions read the exponent
// field only.
template <int I>
__device__ __forceinline__ float row_scale_operand(const uint32_t (&sb)[8])
{
    constexpr int j = I & 3;
    return u2f(j == 3 ? sb[I >> 2] >> 1 : sb[I >> 2] << (23 - 8 * j));
}

// Workgroup -> tile for the transposing kernels.  The hardware deals consecutive workgroup ids
// round-robin to the 8 XCDs, each with its own L2.  Id i therefore takes entry i/8 of XCD (i%8)'s
// own contiguous share of a tile order in which mbm x MBK tiles form a macro block walked
// m-fastest: the tiles an XCD has in flight together are neighbours along m (their output pieces
// and their few-byte scale pieces complete whole lines in that L2) and along k (they share the
// 32-byte sectors of the row scales).  Returns false for the ids that round the grid up.
// mbm is chosen by the launch (macro_block_rows) so that an XCD's share is a whole number of macro
// rows: every XCD then walks its own band of row tiles from the first k tile to the last, all of
// them are at the same k at the same time, and the chip writes whole rows of the output together.
constexpr uint32_t NUM_XCD = 8;
__device__ __forceinline__ bool order_entry_of_workgroup(uint32_t id, uint32_t total, uint32_t *entry)
{
    const uint32_t per_xcd = (total + NUM_XCD - 1) / NUM_XCD;
    *entry = (id % NUM_XCD) * per_xcd + id / NUM_XCD;
    return id / NUM_XCD < per_xcd && *entry < total;
}

// Entry l of the macro-block walk over tiles_m x tiles_k tiles.
template <uint32_t MBK>
__device__ __forceinline__ void tile_of_order_entry(uint32_t l, uint32_t tiles_m, uint32_t tiles_k, uint32_t MBM,
                                                    uint32_t *tile_m, uint32_t *tile_k)
{
    const uint32_t per_macro_row = MBM * tiles_k;
    const uint32_t mg = l / per_macro_row;
    const uint32_t rem = l - mg * per_macro_row;
    const uint32_t mb_rows = min(MBM, tiles_m - mg * MBM);
    const uint32_t kg = rem / (MBK * mb_rows);
    const uint32_t rem2 = rem - kg * MBK * mb_rows;
    const uint32_t k_in = rem2 / mb_rows;
    *tile_m = mg * MBM + (rem2 - k_in * mb_rows);
    *tile_k = kg * MBK + k_in;
}

template <uint32_t MBK>
__device__ __forceinline__ bool tile_of_workgroup(uint32_t id, uint32_t tiles_m, uint32_t tiles_k, uint32_t mbm,
                                                  uint32_t *tile_m, uint32_t *tile_k)
{
    uint32_t l;
    if (!order_entry_of_workgroup(id, tiles_m * tiles_k, &l))
        return false;
    tile_of_order_entry<MBK>(l, tiles_m, tiles_k, mbm, tile_m, tile_k);
    return true;
}

// Row tiles per macro block for a matrix of tiles_m row tiles: an eighth of them, one band per XCD; halved
// while it exceeds 64 (a share is then 2, 4, ... macro rows).  Measured with row_to_col at K = 7168 over rotated
// buffers against a fixed 32: M = 49152 0.63 -> 0.67 of the HBM peak, 61440 0.58 -> 0.67, 73728 0.62 -> 0.685,
// 98304 0.67 -> 0.69; 65536 and 131072 (where an eighth, or a sixteenth, is 32) unchanged; a quarter or a
// sixteenth of the row tiles instead of an eighth: 1-4 % behind wherever they differ from this rule's choice,
// 6-18 % at M = 65536 and 131072.
inline uint32_t macro_block_rows(uint32_t tiles_m)
{
    uint32_t b = (tiles_m + NUM_XCD - 1) / NUM_XCD;
    while (b > 64u)
        b = (b + 1u) / 2u;
    return b ? b : 1u;
}

// Inclusive prefix sum over the 64 lanes of a wave, in the lanes' own registers (DPP): a scan
// inside each row of 16 lanes, then the last lane of row 0 (2) is added to row 1 (3), and lane 31
// to the upper half.
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t v)
{
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, true);  // row_shr:1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, true);  // row_shr:2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, true);  // row_shr:4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, true);  // row_shr:8
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false); // row_bcast:15 -> rows 1, 3
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false); // row_bcast:31 -> rows 2, 3
    return v;
}

// Ragged inputs: workgroup -> (expert, row tile inside it, k tile).  Expert e contributes
// ceil(T_e / TILE_ROWS) row tiles, T_e = off[e+1] - off[e].  The order is expert after expert, each
// expert's tiles in the macro-block walk of tile_of_workgroup over its own row tiles: a macro block
// never spans two experts, whose outputs are separate matrices (a run of m-neighbours that crosses
// into the next expert continues at an unrelated address; measured with a kernel that only moves
// the nibbles of 32 experts of 2048 rows, K = 7168, every byte from and to HBM: 84 us with the
// macro blocks inside the experts, 96 us with 32 concatenated row tiles per block; 83 against 103 us
// at 512 rows per expert).  An expert that extends over several XCD shares gets macro blocks of its width over
// that number (mover: one expert of 61440 rows 95 -> 76 us, two of 30720 81 -> 76, the Zipf-sized and the equal
// experts of the configurations unchanged, three of 21760 82 -> 85).  The XCD shares are cut from this order with the number of tiles that
// really exist (the launch can only bound it: with the bound in its place the ids that round the
// grid up would all fall into the last XCD's share and the others would carry its tiles).
// Uniform per workgroup; every wave evaluates it on its own, 64 experts per lane-parallel step:
// the offsets of all experts (at most 16 x 64) are requested at once, so the lookup waits for
// memory once, then wave prefix sums of the tile counts and a ballot find the expert.
// On success `tile_m` is the tile index inside the expert and, for a non-zero UNIT_A / UNIT_B,
// `a_before` / `b_before` the sum of ceil(T_j / UNIT) over the experts before it (where its
// outputs start when the splits are not padded).
constexpr int MAX_EXPERT_CHUNKS = 16; // 64 experts each: MXFP4_MAX_EXPERTS of the C ABI
template <uint32_t TILE_ROWS, uint32_t UNIT_A, uint32_t UNIT_B, uint32_t MBM_MAX, uint32_t MBK>
__device__ __forceinline__ bool tile_of_grouped_workgroup(const int32_t *off, int32_t num_experts, uint32_t id,
                                                          uint32_t tiles_k, uint32_t *tile_m, uint32_t *tile_k,
                                                          uint32_t *row_base, uint32_t *rows,
                                                          uint32_t *a_before = nullptr, uint32_t *b_before = nullptr)
{
    const uint32_t lane = threadIdx.x & 63u;
    uint32_t lo[MAX_EXPERT_CHUNKS], hi[MAX_EXPERT_CHUNKS];
#pragma unroll
    for (int c = 0; c < MAX_EXPERT_CHUNKS; ++c) {
        lo[c] = hi[c] = 0u;
        if (c * 64 >= num_experts)
            break;
        const int32_t e = c * 64 + (int32_t)lane;
        if (e < num_experts) {
            lo[c] = (uint32_t)off[e];
            hi[c] = (uint32_t)off[e + 1];
        }
    }
    uint32_t total = 0; // row tiles of all experts
    uint32_t incl[MAX_EXPERT_CHUNKS]; // prefix sums of the tile counts inside each chunk
#pragma unroll
    for (int c = 0; c < MAX_EXPERT_CHUNKS; ++c) {
        incl[c] = 0u;
        if (c * 64 >= num_experts)
            break;
        incl[c] = wave_inclusive_sum((hi[c] - lo[c] + TILE_ROWS - 1u) / TILE_ROWS);
        total += (uint32_t)__builtin_amdgcn_readlane((int)incl[c], 63);
    }
    uint32_t entry;
    if (!order_entry_of_workgroup(id, total * tiles_k, &entry))
        return false;
    const uint32_t tile = entry / tiles_k; // the expert whose row tiles include this index holds the entry

    uint32_t before = 0, abefore = 0, bbefore = 0; // tiles / units of the experts in earlier chunks
#pragma unroll
    for (int c = 0; c < MAX_EXPERT_CHUNKS; ++c) {
        if (c * 64 >= num_experts)
            break;
        const uint32_t len = hi[c] - lo[c];
        const uint32_t nt = (len + TILE_ROWS - 1u) / TILE_ROWS;
        const uint32_t na = UNIT_A ? (len + UNIT_A - 1u) / (UNIT_A ? UNIT_A : 1u) : 0u;
        const uint32_t nb = UNIT_B ? (len + UNIT_B - 1u) / (UNIT_B ? UNIT_B : 1u) : 0u;
        const uint32_t aincl = UNIT_A ? wave_inclusive_sum(na) : 0u;
        const uint32_t bincl = UNIT_B ? wave_inclusive_sum(nb) : 0u;
        const uint64_t hit = __ballot(before + incl[c] > tile);
        if (hit != 0ull) {
            const int l = __ffsll((unsigned long long)hit) - 1;
            const uint32_t excl = (uint32_t)__builtin_amdgcn_readlane((int)(incl[c] - nt), l);
            *row_base = (uint32_t)__builtin_amdgcn_readlane((int)lo[c], l);
            *rows = (uint32_t)__builtin_amdgcn_readlane((int)len, l);
            const uint32_t nt_e = (uint32_t)__builtin_amdgcn_readlane((int)nt, l);
            // macro block: the expert's width over the number of XCD shares it extends over (one expert is
            // then walked like a single matrix, see macro_block_rows), halved while above MBM_MAX
            // (the divisions only for an expert of at least 1.5 shares)
            uint32_t mbm = nt_e;
            if (2u * NUM_XCD * nt_e >= 3u * total) {
                const uint32_t spans = (NUM_XCD * nt_e + total / 2u) / total;
                mbm = (nt_e + spans - 1u) / spans;
            }
            while (mbm > MBM_MAX)
                mbm = (mbm + 1u) / 2u;
            tile_of_order_entry<MBK>(entry - (before + excl) * tiles_k, nt_e, tiles_k, mbm, tile_m, tile_k);
            if (UNIT_A)
                *a_before = abefore + (uint32_t)__builtin_amdgcn_readlane((int)(aincl - na), l);
            if (UNIT_B)
                *b_before = bbefore + (uint32_t)__builtin_amdgcn_readlane((int)(bincl - nb), l);
            return true;
        }
        before += (uint32_t)__builtin_amdgcn_readlane((int)incl[c], 63);
        if (UNIT_A)
            abefore += (uint32_t)__builtin_amdgcn_readlane((int)aincl, 63);
        if (UNIT_B)
            bbefore += (uint32_t)__builtin_amdgcn_readlane((int)bincl, 63);
    }
    return false; // not reached: tile < total
}

// Streaming stores for outputs that this kernel does not read again: the non-temporal hint together
// with the sc1 bit of the gfx940-family vector stores (the write goes through at device scope
// instead of waiting in the L2 for an eviction).  Measured at [65536,7168] with every byte going to HBM:
// the 16-byte E4M3 stores of the de-quantizer, written in address order by the whole grid, 115 -> 111 us
// against the non-temporal hint alone.  Where neighbouring workgroups complete each other's lines (the
// transposed rows of row_to_col: 93 -> 97 us) or the pieces are small, the hint alone is the better form.
// The builtin non-temporal store only sets the hint, hence the asm.
__device__ __forceinline__ void store_streaming(void *p, u32x4 v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc1 nt" : : "v"(p), "v"(v) : "memory");
}

// The first n (1..15) bytes of v to dst, any alignment, in at most four pieces.
__device__ __forceinline__ void store_head_bytes(uint8_t *dst, const u32x4 v, uint32_t n)
{
    uint32_t pos = 0; // bytes done
    if (n & 8u) {
        *reinterpret_cast<u64_unaligned *>(dst) = ((uint64_t)v.y << 32) | v.x;
        pos = 8;
    }
    if (n & 4u) {
        *reinterpret_cast<u32_unaligned *>(dst + pos) = pos ? v.z : v.x;
        pos += 4;
    }
    const uint32_t d = pos == 0u ? v.x : pos == 4u ? v.y : pos == 8u ? v.z : v.w; // the dword still open
    if (n & 2u)
        *reinterpret_cast<u16_unaligned *>(dst + pos) = (uint16_t)d;
    if (n & 1u)
        dst[pos + (n & 2u)] = (uint8_t)(d >> (8u * (n & 2u)));
}

// Compile-time loop: f(std::integral_constant<int, 0>) ... f(std::integral_constant<int, N-1>).
// The conversion builtins take their byte selector as an immediate.
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(static_cast<F &&>(f), std::make_integer_sequence<int, N>{});
}

} // namespace mxfp4
