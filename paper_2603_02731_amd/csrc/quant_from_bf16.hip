// BF16 -> MXFP4 (packed E2M1 + UE8M0 per 1x32), gfx950: the row-wise quantizer exactly as the
// paper states it (sec. 3.1, BF16ToFP4Row): SF = 2^ceil(log2(group_max / 6)) per 1x32 block,
// then RTNE onto E2M1.  A BF16 value is the upper half of an FP32, so widening is a shift and
// everything after it is the same as in the FP8-source kernel.
//
// Work split: one lane owns 8 consecutive elements (one 16-byte load), so a block of 32 is 4
// lanes and 16 lanes hold the 4 blocks whose scale bytes form one aligned dword.  Per lane:
//   16 B load -> 8 shifts/masks -> NaN-propagating |max| -> two DPP exchanges inside the quad
//   -> exponent-field arithmetic for the UE8M0 byte -> 4 x v_cvt_scalef32_pk_fp4_f32
//   -> one dword store of 8 nibbles; lane 0 of every 16 stores the 4 scale bytes as a dword.
// HBM-bound: 2 B read + 0.53125 B written per element.
#include "mxfp4_device.hpp"
#include "mxfp4_kernels.hpp"

namespace mxfp4 {

// store_streaming instead of the non-temporal hint: 185 -> 186 us at [65536,7168], not used.

constexpr int QBF_THREADS = 512; // 512 lanes x 2 runs: 182-184 us at [65536,7168], 256 x 2 185, 1024 x 2 189, one run per lane 193-218
constexpr int QBF_UNROLL = 2;

struct QuantBf16Args {
    const uint16_t *x;
    uint8_t *q;
    uint8_t *sf;
    int64_t ld_q;
    int64_t ld_sf;
    uint32_t n_chunks;       // M * K / 8
    uint32_t chunks_per_row; // K / 8
};

template <bool DENSE>
__global__ void __launch_bounds__(QBF_THREADS) quant_from_bf16_kernel(const QuantBf16Args a)
{
    const uint32_t c0 = blockIdx.x * (QBF_THREADS * QBF_UNROLL) + threadIdx.x;

    u32x4 w[QBF_UNROLL];
#pragma unroll
    for (int u = 0; u < QBF_UNROLL; ++u) {
        const uint32_t c = c0 + u * QBF_THREADS;
        if (c >= a.n_chunks)
            break; // n_chunks is a multiple of 16: the 16 lanes of a scale dword leave together
        w[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.x + (size_t)c * 8));
    }

#pragma unroll
    for (int u = 0; u < QBF_UNROLL; ++u) {
        const uint32_t c = c0 + u * QBF_THREADS;
        if (c >= a.n_chunks)
            break;
        float v[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v[2 * j] = u2f(w[u][j] << 16);
            v[2 * j + 1] = u2f(w[u][j] & 0xFFFF0000u);
        }
        float m = 0.0f;
#pragma unroll
        for (int j = 0; j < 8; j += 2)
            m = max3_abs_nan(v[j], v[j + 1], m);
        m = __builtin_elementwise_maximum(m, u2f(dpp_read<DPP_QUAD_XOR1>(f2u(m))));
        m = __builtin_elementwise_maximum(m, u2f(dpp_read<DPP_QUAD_XOR2>(f2u(m))));

        const uint32_t b = ue8m0_of_block_max(f2u(m));
        const float sc = u2f(b << 23); // only the exponent field of the scale operand is used
        uint32_t r = 0;
        r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, v[0], v[1], sc, 0);
        r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, v[2], v[3], sc, 1);
        r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, v[4], v[5], sc, 2);
        r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, v[6], v[7], sc, 3);
        r = b == 255u ? 0u : r; // a NaN poisons the block: codes are zeroed

        uint8_t *dst_q, *dst_sf;
        if (DENSE) {
            dst_q = a.q + (size_t)c * 4;
            dst_sf = a.sf + (size_t)(c >> 4) * 4;
        } else {
            const uint32_t row = c / a.chunks_per_row;
            const uint32_t cc = c - row * a.chunks_per_row;
            dst_q = a.q + (size_t)row * a.ld_q + (size_t)cc * 4;
            dst_sf = a.sf + (size_t)row * a.ld_sf + (size_t)(cc >> 4) * 4;
        }
        __builtin_nontemporal_store(r, reinterpret_cast<uint32_t *>(dst_q));

        // lanes 4j..4j+3 of a row of 16 hold block j's byte: gather the four into lane 0
        uint32_t t = b | (row_shift_left4(b) << 8); // lanes 0..3: B0 | B1 << 8; lanes 8..11: B2 | B3 << 8
        t |= row_shift_left8(t) << 16;
        if ((threadIdx.x & 15u) == 0u)
            *reinterpret_cast<uint32_t *>(dst_sf) = t;
    }
}

hipError_t launch_quant_from_bf16(const uint16_t *x, int64_t M, int64_t K, uint8_t *q, int64_t ld_q, uint8_t *sf,
                                  int64_t ld_sf, hipStream_t stream)
{
    QuantBf16Args a;
    a.x = x;
    a.q = q;
    a.sf = sf;
    a.ld_q = ld_q;
    a.ld_sf = ld_sf;
    a.n_chunks = (uint32_t)(M * (K / 8));
    a.chunks_per_row = (uint32_t)(K / 8);
    constexpr uint32_t per_block = QBF_THREADS * QBF_UNROLL;
    const uint32_t blocks = (a.n_chunks + per_block - 1) / per_block;
    if (ld_q == K / 2 && ld_sf == K / 32)
        hipLaunchKernelGGL(quant_from_bf16_kernel<true>, dim3(blocks), dim3(QBF_THREADS), 0, stream, a);
    else
        hipLaunchKernelGGL(quant_from_bf16_kernel<false>, dim3(blocks), dim3(QBF_THREADS), 0, stream, a);
    return hipGetLastError();
}

} // namespace mxfp4
