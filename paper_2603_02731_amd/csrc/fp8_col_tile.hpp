// Pieces shared by the two row-blocked MXFP4 -> column-wise FP8 kernels (scale alignment and
// re-quantization): the write-out of a finished 256-column tile part from LDS to the [K, rows]
// byte matrix of one expert, ragged ends and unaligned rows included.
#pragma once

#include "mxfp4_device.hpp"

namespace mxfp4 {
namespace fp8col {

typedef short s16x2 __attribute__((ext_vector_type(2)));

// Write the finished tile out of LDS: 16 lanes per k-row, 256 contiguous bytes, 256 lanes.  LDS row
// c*32 + cg is column 8*cg + c of the tile, as 16 slots of 16 bytes, the slot of rows 16*l.. being
// (l + cg) % 16.  Chunk u*256 + tid of the tile is row c*32 + cgx, physical slot tid%16, with
// cgx = tid/16 in the even passes and tid/16 + 16 in the odd ones.
// krow0 = address of k-row 0, byte m0 of the expert's matrix; uniform k-row pointers plus
// one 32-bit lane offset (M <= 2^24).  n_rows = rows of the tile that exist (1..256).
// store_streaming instead of the non-temporal hint: 128 -> 139 us at [65536,7168].  The 256-byte pieces of
// neighbouring tiles are better merged in the caches than written through one by one.
__device__ __forceinline__ void write_tile_out(const u32x4 *s_out, uint8_t *krow0, const uint8_t *out_x, size_t pitch_x,
                                               uint32_t cols, uint32_t n_rows, uint32_t tid)
{
    constexpr int CP = 8, T = 256, HALVES = 2; // columns per lane, lanes, passes per column
    const uint32_t pslot = tid & 15u;
    const uint32_t lslot = (pslot - (tid >> 4)) & 15u; // 16 bytes = rows 16*lslot.. of the tile
    const uint32_t lane_off = (tid >> 4) * 8u * (uint32_t)pitch_x + lslot * 16u;
    // Rows on 64-byte boundaries (always, unless the splits are ragged) leave with non-temporal
    // stores.  The others leave with plain, possibly unaligned vector stores and the L2 merges
    // the pieces of neighbouring tiles: measured with 32 un-padded experts at [61440,7168]
    // 204 us, against 258 us with non-temporal stores and 286 us with the rows realigned in
    // registers (funnel shift of neighbouring 16-byte pieces, every store naturally aligned).
    // A tile's 256-byte piece of a k-row must consist of whole 64-byte segments for the
    // streaming form to pay: 32 experts of 1824 rows (32-byte boundaries) take 184 us with it
    // and about 162 us without, 1856 rows (64-byte boundaries) 142 us with it.
    const bool streaming = ((reinterpret_cast<uintptr_t>(out_x) | pitch_x) & 63u) == 0u;
    // bytes of this lane's 16-byte piece that exist: 16, or fewer at the ragged end of a split
    const uint32_t have = lslot * 16u < n_rows ? min(16u, n_rows - lslot * 16u) : 0u;
    static_for<HALVES>([&](auto oddp) {
        constexpr int odd = decltype(oddp)::value;
        if ((odd * 16u + (tid >> 4)) * 8u < cols && have != 0u) {
            if (have == 16u && streaming) {
#pragma unroll
                for (int c = 0; c < CP; ++c) {
                    uint8_t *dst = krow0 + (size_t)(odd * 128u + c) * pitch_x + lane_off;
                    __builtin_nontemporal_store(s_out[(HALVES * c + odd) * T + tid], reinterpret_cast<u32x4 *>(dst));
                }
            } else if (have == 16u) {
                // any alignment: global memory takes unaligned vector stores
#pragma unroll
                for (int c = 0; c < CP; ++c) {
                    uint8_t *dst = krow0 + (size_t)(odd * 128u + c) * pitch_x + lane_off;
                    *reinterpret_cast<u32x4_unaligned *>(dst) = s_out[(HALVES * c + odd) * T + tid];
                }
            } else {
#pragma nounroll
                for (int c = 0; c < CP; ++c) {
                    uint8_t *dst = krow0 + (size_t)(odd * 128u + c) * pitch_x + lane_off;
                    store_head_bytes(dst, s_out[(HALVES * c + odd) * T + tid], have);
                }
            }
        }
    });
}

} // namespace fp8col
} // namespace mxfp4
