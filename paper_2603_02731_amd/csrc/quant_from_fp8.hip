// FP8 (E4M3 + FP32 1x128 scales) -> MXFP4 (packed E2M1 + UE8M0 per 1x32), gfx950.
//
// Paper sec. 3.1: SF = 2^ceil(log2(group_max / 6)) per 1x32 block, then RTNE onto E2M1.
// The element values are the FP8 values themselves, fl32(e4m3 * tile scale): nothing
// passes through BF16 (the direct FP8 -> FP4 path of the paper's contributions).
//
// Work split: one lane owns 16 consecutive elements (one 16-byte load), so a block of 32
// is a pair of lanes and a 128-tile is 8 lanes.  Per lane:
//   16 B load -> 8 x v_cvt_pk_f32_fp8 -> 16 x v_mul_f32 (the one FP32 rounding)
//   -> NaN-propagating |max| (v_maximum3_f32) -> one DPP exchange with the pair lane
//   -> exponent-field arithmetic for the UE8M0 byte -> 8 x v_cvt_scalef32_pk_fp4_f32
//   -> one 8-byte store of 16 nibbles; the tile's four scale bytes are gathered by DPP
//      into lane 0 of its 8 lanes and leave as one dword.
// HBM-bound: 1.03125 B read + 0.53125 B written per element.
#include "mxfp4_device.hpp"
#include "mxfp4_kernels.hpp"

namespace mxfp4 {

// Lanes per workgroup (each lane takes QUANT_UNROLL chunks).  Dense rows: 512 x 2 runs; at [65536,7168] over
// rotated buffers 256 x 2 and 256 x 4 are as fast, 1024 x 2 is 5 % slower.  Gathered, strided and scattered rows: 256.
constexpr int QUANT_THREADS = 512;        // dense rows
constexpr int QUANT_THREADS_ROUTED = 256; // gathered, strided, scattered rows
constexpr int QUANT_UNROLL = 2;
// Cache policy, measured at [65536,7168] over rotated buffer sets (every byte from and to HBM): non-temporal
// loads and stores 109 us; non-temporal loads with plain stores 118 us (that form is the faster one, 104 against
// 107 us, only when the 250 MB of output are rewritten in place and stay in the memory-side cache); plain
// loads 121 us.  Gathered rows are read several times: plain loads with non-temporal stores 1012 us for the
// top-8 payload of 65536 tokens, plain both ways 1090 us, non-temporal loads with plain stores 1130 us.

struct QuantArgs {
    const uint8_t *x;
    const float *x_scale;
    const int32_t *gather_idx;
    uint8_t *q;
    uint8_t *sf;
    int64_t ld_q;
    int64_t ld_sf;
    uint32_t n_chunks;       // M_out * K / 16
    uint32_t chunks_per_row; // K / 16
    uint32_t K;
    uint32_t M_src;
};

// Quantize the lane's 16 elements given as four dwords of E4M3 bytes and the tile scale.
// Returns the 16 nibbles in out[0..1]; *scale_byte is the block's UE8M0 byte (identical
// in both lanes of the pair).
__device__ __forceinline__ void quant16(const u32x4 w, float s, uint32_t out[2], uint32_t *scale_byte)
{
    float v[16];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8(w[j], false);
        f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8(w[j], true);
        v[4 * j + 0] = lo.x * s;
        v[4 * j + 1] = lo.y * s;
        v[4 * j + 2] = hi.x * s;
        v[4 * j + 3] = hi.y * s;
    }
    float m = 0.0f;
#pragma unroll
    for (int j = 0; j < 16; j += 2)
        m = max3_abs_nan(v[j], v[j + 1], m);
    float other = u2f(dpp_read<DPP_QUAD_XOR1>(f2u(m)));
    m = __builtin_elementwise_maximum(m, other);

    uint32_t b = ue8m0_of_block_max(f2u(m));
    float sc = u2f(b << 23); // only the exponent field of the scale operand is used
    uint32_t r0 = 0, r1 = 0;
    r0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r0, v[0], v[1], sc, 0);
    r0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r0, v[2], v[3], sc, 1);
    r0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r0, v[4], v[5], sc, 2);
    r0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r0, v[6], v[7], sc, 3);
    r1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r1, v[8], v[9], sc, 0);
    r1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r1, v[10], v[11], sc, 1);
    r1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r1, v[12], v[13], sc, 2);
    r1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r1, v[14], v[15], sc, 3);
    const bool nan_block = b == 255u; // a NaN poisons the block: codes are zeroed
    out[0] = nan_block ? 0u : r0;
    out[1] = nan_block ? 0u : r1;
    *scale_byte = b;
}

// store_streaming instead of the non-temporal hint, measured at [65536,7168] on one buffer set: the 8-byte nibble stores of the
// dense kernel 112.0 -> 112.1 us (no difference), its scale dwords 112 -> 121 us, the scattered rows
// 463 -> 466 us, gathered per-token records 1065 -> 1400 us: not used here.
//
// One workgroup covers QUANT_UNROLL runs of THREADS consecutive chunks; a lane takes chunk
// `tid` of each run, so every load and store instruction of a wave stays contiguous
// (1 KiB in, 512 B out) while each lane keeps QUANT_UNROLL loads in flight.
// DENSE: no gather and dense outputs -- every address is a multiple of the flat chunk index.
template <bool DENSE, bool GATHER, int THREADS>
__global__ void __launch_bounds__(THREADS) quant_from_fp8_kernel(const QuantArgs a)
{
    const uint32_t c0 = blockIdx.x * (THREADS * QUANT_UNROLL) + threadIdx.x;

    u32x4 w[QUANT_UNROLL];
    float s[QUANT_UNROLL];
    uint8_t *dst_q[QUANT_UNROLL];
    uint8_t *dst_sf[QUANT_UNROLL]; // the tile's four scale bytes (one aligned dword)
#pragma unroll
    for (int u = 0; u < QUANT_UNROLL; ++u) {
        const uint32_t c = c0 + u * THREADS;
        if (c >= a.n_chunks)
            break; // n_chunks is a multiple of 8: the 8 lanes of a tile leave together
        const uint8_t *src;
        const float *src_scale;
        bool valid = true;
        if (DENSE) {
            src = a.x + (size_t)c * 16;
            src_scale = a.x_scale + (c >> 3);
            dst_q[u] = a.q + (size_t)c * 8;
            dst_sf[u] = a.sf + (size_t)(c >> 3) * 4;
        } else {
            const uint32_t row = c / a.chunks_per_row;
            const uint32_t cc = c - row * a.chunks_per_row;
            uint32_t src_row = row;
            if (GATHER) {
                src_row = (uint32_t)a.gather_idx[row];
                valid = src_row < a.M_src; // also rejects negative indices
                src_row = valid ? src_row : 0u;
            }
            src = a.x + (size_t)src_row * a.K + (size_t)cc * 16;
            src_scale = a.x_scale + (size_t)src_row * (a.K >> 7) + (cc >> 3);
            dst_q[u] = a.q + (size_t)row * a.ld_q + (size_t)cc * 8;
            dst_sf[u] = a.sf + (size_t)row * a.ld_sf + (size_t)(cc >> 3) * 4;
        }
        if (!GATHER)
            w[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src));
        else
            w[u] = *reinterpret_cast<const u32x4 *>(src); // gathered rows are read several times
        s[u] = *src_scale;
        if (!valid) { // an out-of-range gather index yields a zero row
            w[u] = u32x4{0u, 0u, 0u, 0u};
            s[u] = 0.0f;
        }
    }

#pragma unroll
    for (int u = 0; u < QUANT_UNROLL; ++u) {
        if (c0 + u * THREADS >= a.n_chunks)
            break;
        uint32_t out[2], b;
        quant16(w[u], s[u], out, &b);
        __builtin_nontemporal_store(u32x2{out[0], out[1]}, reinterpret_cast<u32x2 *>(dst_q[u]));

        // lanes 2j, 2j+1 of the tile's 8 hold block j's byte: gather the four into lane 0
        uint32_t t = b | (dpp_read<DPP_QUAD_XOR2>(b) << 8); // lanes 0,1: B0 | B1 << 8
        t |= row_shift_left4(t) << 16;                       // lane 0: ... | B2 << 16 | B3 << 24
        if ((threadIdx.x & 7u) == 0u) {
            *reinterpret_cast<uint32_t *>(dst_sf[u]) = t;
        }
    }
}

// The routing turned around: every source row is read and quantized once and written to each of
// its `fanout` destination rows (a token and its top-k experts), instead of being read and
// quantized again for every destination.  Same lane layout; dense source, strided outputs.
struct QuantScatterArgs {
    const uint8_t *x;
    const float *x_scale;
    const int32_t *dst_idx; // [M_src, fanout]
    uint8_t *q;
    uint8_t *sf;
    int64_t ld_q;
    int64_t ld_sf;
    uint32_t n_chunks;       // M_src * K / 16
    uint32_t chunks_per_row; // K / 16
    uint32_t fanout;
    uint32_t M_out;
};

__global__ void __launch_bounds__(QUANT_THREADS_ROUTED) quant_from_fp8_scatter_kernel(const QuantScatterArgs a)
{
    const uint32_t c0 = blockIdx.x * (QUANT_THREADS_ROUTED * QUANT_UNROLL) + threadIdx.x;

    u32x4 w[QUANT_UNROLL];
    float s[QUANT_UNROLL];
#pragma unroll
    for (int u = 0; u < QUANT_UNROLL; ++u) {
        const uint32_t c = c0 + u * QUANT_THREADS_ROUTED;
        if (c >= a.n_chunks)
            break; // n_chunks is a multiple of 8: the 8 lanes of a tile leave together
        w[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.x + (size_t)c * 16));
        s[u] = a.x_scale[c >> 3];
    }

#pragma unroll
    for (int u = 0; u < QUANT_UNROLL; ++u) {
        const uint32_t c = c0 + u * QUANT_THREADS_ROUTED;
        if (c >= a.n_chunks)
            break;
        uint32_t out[2], b;
        quant16(w[u], s[u], out, &b);
        // lanes 2j, 2j+1 of the tile's 8 hold block j's byte: gather the four into lane 0
        uint32_t t = b | (dpp_read<DPP_QUAD_XOR2>(b) << 8); // lanes 0,1: B0 | B1 << 8
        t |= row_shift_left4(t) << 16;                       // lane 0: ... | B2 << 16 | B3 << 24

        const uint32_t row = c / a.chunks_per_row;
        const uint32_t cc = c - row * a.chunks_per_row;
        const int32_t *dst = a.dst_idx + (size_t)row * a.fanout;
        // the destinations are read eight at a time before any store: a store (bytes, may alias
        // anything) between two index loads would put every load's latency on the lane's path
        for (uint32_t j0 = 0; j0 < a.fanout; j0 += 8u) {
            uint32_t d[8];
#pragma unroll
            for (int j = 0; j < 8; ++j)
                d[j] = j0 + j < a.fanout ? (uint32_t)dst[j0 + j] : 0xFFFFFFFFu;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (d[j] >= a.M_out) // also skips negative entries and the tail of the batch
                    continue;
                __builtin_nontemporal_store(u32x2{out[0], out[1]},
                                            reinterpret_cast<u32x2 *>(a.q + (size_t)d[j] * a.ld_q + (size_t)cc * 8));
                if ((threadIdx.x & 7u) == 0u)
                    *reinterpret_cast<uint32_t *>(a.sf + (size_t)d[j] * a.ld_sf + (size_t)(cc >> 3) * 4) = t;
            }
        }
    }
}

// The scatter form for 16-byte-aligned outputs: a workgroup quantizes SCATTER_ROWS whole source rows into LDS
// (per row the K/2 nibble bytes followed by the K/32 scale bytes, as they sit in a per-token record) and
// then writes every row to each of its destinations in 16-byte pieces, whole rows contiguous: one wave
// instruction stores 1 KiB of one destination row, and the scale bytes leave in the same stream instead of
// as scattered dwords.
// The destination indices of a row are uniform over the workgroup.
constexpr int SCATTER_ROWS = 4; // at most; the launcher picks 1, 2 or 4 rows per workgroup
constexpr int SCATTER_THREADS = 512;
constexpr int SCATTER_UNROLL = 1;

template <bool WIDE_SF> // the K/32 scale bytes of a row are a whole number of 16-byte pieces (K % 512 == 0)
__global__ void __launch_bounds__(SCATTER_THREADS) quant_from_fp8_scatter_rows_kernel(const QuantScatterArgs a,
                                                                                      const uint32_t M_src,
                                                                                      const uint32_t rows_per_wg)
{
    extern __shared__ __align__(16) uint8_t s_rows[]; // [SCATTER_ROWS][rec], rec = K/2 + K/32 rounded up to 16
    const uint32_t tid = threadIdx.x;
    const uint32_t C = a.chunks_per_row;              // 16-element chunks per row
    const uint32_t nib_bytes = C * 8u, sf_bytes = C / 2u;
    const uint32_t rec = (nib_bytes + sf_bytes + 15u) & ~15u;
    const uint32_t row0 = blockIdx.x * rows_per_wg;
    const uint32_t n_rows = min(rows_per_wg, M_src - row0);
    const uint32_t n_chunks = n_rows * C;             // a multiple of 8
    const uint8_t *src = a.x + (size_t)row0 * C * 16u;
    const float *src_scale = a.x_scale + (size_t)row0 * (C / 8u);

    // the first eight destinations of every row, requested before anything else (uniform over the workgroup)
    uint32_t dpre[SCATTER_ROWS][8];
#pragma unroll
    for (int r = 0; r < SCATTER_ROWS; ++r)
#pragma unroll
        for (int j = 0; j < 8; ++j)
            dpre[r][j] = (uint32_t)r < n_rows && (uint32_t)j < a.fanout
                             ? (uint32_t)a.dst_idx[(size_t)(row0 + r) * a.fanout + j]
                             : 0xFFFFFFFFu;

    for (uint32_t base = 0; base < n_chunks; base += SCATTER_THREADS * SCATTER_UNROLL) {
        u32x4 w[SCATTER_UNROLL];
        float s[SCATTER_UNROLL];
#pragma unroll
        for (int u = 0; u < SCATTER_UNROLL; ++u) {
            const uint32_t c = base + u * SCATTER_THREADS + tid;
            if (c < n_chunks) { // the 8 lanes of a tile pass or fail together
                w[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + (size_t)c * 16u));
                s[u] = src_scale[c >> 3];
            }
        }
#pragma unroll
        for (int u = 0; u < SCATTER_UNROLL; ++u) {
            const uint32_t c = base + u * SCATTER_THREADS + tid;
            if (c < n_chunks) {
                uint32_t out[2], b;
                quant16(w[u], s[u], out, &b);
                uint32_t t = b | (dpp_read<DPP_QUAD_XOR2>(b) << 8); // lanes 0,1 of the tile: B0 | B1 << 8
                t |= row_shift_left4(t) << 16;                       // lane 0: ... | B2 << 16 | B3 << 24
                const uint32_t r = c / C, cc = c - r * C;
                uint8_t *row = s_rows + r * rec;
                *reinterpret_cast<u32x2 *>(row + cc * 8u) = u32x2{out[0], out[1]};
                if ((tid & 7u) == 0u)
                    *reinterpret_cast<uint32_t *>(row + nib_bytes + (cc >> 3) * 4u) = t;
            }
        }
    }
    __syncthreads();

    const uint32_t nib_pieces = nib_bytes / 16u;
    const uint32_t sf_pieces = WIDE_SF ? sf_bytes / 16u : sf_bytes / 4u; // 16-byte pieces, or dwords
    // the scale pieces go to the lanes after those of the last nibble pieces
    const uint32_t sf_lane = (tid + SCATTER_THREADS - nib_pieces % SCATTER_THREADS) % SCATTER_THREADS;
    auto store_row = [&](uint32_t r, uint32_t d) {
        if (d >= a.M_out) // also skips negative entries and the slots past the fan-out
            return;
        const uint8_t *row = s_rows + r * rec;
        uint8_t *dq = a.q + (size_t)d * a.ld_q;
        uint8_t *dsf = a.sf + (size_t)d * a.ld_sf;
        for (uint32_t p = tid; p < nib_pieces; p += SCATTER_THREADS)
            __builtin_nontemporal_store(*reinterpret_cast<const u32x4 *>(row + p * 16u),
                                        reinterpret_cast<u32x4 *>(dq + p * 16u));
        for (uint32_t p = sf_lane; p < sf_pieces; p += SCATTER_THREADS) {
            if (WIDE_SF)
                __builtin_nontemporal_store(*reinterpret_cast<const u32x4 *>(row + nib_bytes + p * 16u),
                                            reinterpret_cast<u32x4 *>(dsf + p * 16u));
            else
                *reinterpret_cast<uint32_t *>(dsf + p * 4u) = *reinterpret_cast<const uint32_t *>(row + nib_bytes + p * 4u);
        }
    };
#pragma unroll
    for (int r = 0; r < SCATTER_ROWS; ++r) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
            store_row(r, dpre[r][j]);
        if ((uint32_t)r < n_rows) {
            const int32_t *dst = a.dst_idx + (size_t)(row0 + r) * a.fanout;
            for (uint32_t j = 8; j < a.fanout; ++j) // fan-outs beyond 8: one index at a time
                store_row(r, (uint32_t)dst[j]);
        }
    }
}

hipError_t launch_quant_from_fp8_scatter(const uint8_t *x, const float *x_scale, int64_t M_src, int64_t K,
                                         const int32_t *dst_idx, int32_t fanout, int64_t M_out, uint8_t *q,
                                         int64_t ld_q, uint8_t *sf, int64_t ld_sf, hipStream_t stream)
{
    QuantScatterArgs a;
    a.x = x;
    a.x_scale = x_scale;
    a.dst_idx = dst_idx;
    a.q = q;
    a.sf = sf;
    a.ld_q = ld_q;
    a.ld_sf = ld_sf;
    a.n_chunks = (uint32_t)(M_src * (K / 16));
    a.chunks_per_row = (uint32_t)(K / 16);
    a.fanout = (uint32_t)fanout;
    a.M_out = (uint32_t)M_out;
    // whole rows through LDS when every output row starts on a 16-byte boundary and four rows fit into LDS
    const uint32_t rec = (uint32_t)((K / 2 + K / 32 + 15) & ~(int64_t)15);
    const bool rows16 = ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(sf) | (uintptr_t)ld_q |
                          (uintptr_t)ld_sf) & 15u) == 0u;
    if (rows16 && rec <= 48u * 1024u) {
        // Rows per workgroup: about one 16-element chunk per lane.  Top-8 payload of 65536 tokens at K = 7168 into
        // 3808-byte records, over rotated buffers, destinations shuffled / in token order: 512 lanes x 1 chunk, one
        // row 552 / 427 us; 256 lanes x 4 chunks, one row 545 / 458, four rows 588 / 545; two rows on 896 lanes
        // 597 / 559 (more, shorter workgroups overlap their loads, stores and the wait for the last store better).
        // The kernel it replaces, with 8-byte nibble stores and the scale dwords on their own: 598 us shuffled.
        // With shuffled destinations the records bound it: 3808 bytes are 29.75 lines, so both ends of every
        // record are partial lines written by different workgroups (planes of 3584 + 224 bytes: 516 us; a kernel
        // that only copies 16 bytes per lane to eight destination streams: 395-430 us).
        const uint32_t C = a.chunks_per_row;
        const uint32_t rows = 2u * C >= SCATTER_THREADS ? 1u : 4u * C >= SCATTER_THREADS ? 2u : 4u;
        const uint32_t blocks = (uint32_t)((M_src + rows - 1) / rows);
        if (K % 512 == 0)
            hipLaunchKernelGGL(quant_from_fp8_scatter_rows_kernel<true>, dim3(blocks), dim3(SCATTER_THREADS),
                               rows * rec, stream, a, (uint32_t)M_src, rows);
        else
            hipLaunchKernelGGL(quant_from_fp8_scatter_rows_kernel<false>, dim3(blocks), dim3(SCATTER_THREADS),
                               rows * rec, stream, a, (uint32_t)M_src, rows);
        return hipGetLastError();
    }
    constexpr uint32_t per_block = QUANT_THREADS_ROUTED * QUANT_UNROLL;
    const uint32_t blocks = (a.n_chunks + per_block - 1) / per_block;
    hipLaunchKernelGGL(quant_from_fp8_scatter_kernel, dim3(blocks), dim3(QUANT_THREADS_ROUTED), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_quant_from_fp8(const uint8_t *x, const float *x_scale, int64_t M_src, int64_t K,
                                 const int32_t *gather_idx, int64_t M_out, uint8_t *q, int64_t ld_q,
                                 uint8_t *sf, int64_t ld_sf, hipStream_t stream)
{
    QuantArgs a;
    a.x = x;
    a.x_scale = x_scale;
    a.gather_idx = gather_idx;
    a.q = q;
    a.sf = sf;
    a.ld_q = ld_q;
    a.ld_sf = ld_sf;
    a.n_chunks = (uint32_t)(M_out * (K / 16));
    a.chunks_per_row = (uint32_t)(K / 16);
    a.K = (uint32_t)K;
    a.M_src = (uint32_t)M_src;
    const bool dense = gather_idx == nullptr && ld_q == K / 2 && ld_sf == K / 32;
    const uint32_t per_block = (dense ? QUANT_THREADS : QUANT_THREADS_ROUTED) * QUANT_UNROLL;
    const uint32_t blocks = (a.n_chunks + per_block - 1) / per_block;
    if (dense)
        hipLaunchKernelGGL((quant_from_fp8_kernel<true, false, QUANT_THREADS>), dim3(blocks), dim3(QUANT_THREADS), 0,
                           stream, a);
    else if (gather_idx)
        hipLaunchKernelGGL((quant_from_fp8_kernel<false, true, QUANT_THREADS_ROUTED>), dim3(blocks),
                           dim3(QUANT_THREADS_ROUTED), 0, stream, a);
    else
        hipLaunchKernelGGL((quant_from_fp8_kernel<false, false, QUANT_THREADS_ROUTED>), dim3(blocks),
                           dim3(QUANT_THREADS_ROUTED), 0, stream, a);
    return hipGetLastError();
}

} // namespace mxfp4
