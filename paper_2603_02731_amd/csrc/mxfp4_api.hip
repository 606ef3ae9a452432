// The C ABI of libmxfp4 (include/mxfp4.h): argument validation and kernel launches.
// Nothing here allocates, copies or synchronises.
#include "../../include/mxfp4.h"
#include "mxfp4_device.hpp"
#include "mxfp4_kernels.hpp"

namespace {

inline bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

inline mxfp4_status launched(hipError_t e) { return e == hipSuccess ? MXFP4_OK : MXFP4_ERR_LAUNCH; }

constexpr int64_t kMaxWorkItems = ((int64_t)1 << 32) - 4096; // kernels index their work with 32 bits
constexpr int64_t kMaxRows = (int64_t)1 << 31;
static_assert(mxfp4::MAX_EXPERT_CHUNKS * 64 >= MXFP4_MAX_EXPERTS, "the expert lookup of the grouped kernels holds every expert's offsets");

} // namespace

namespace mxfp4 {

uint32_t compute_units()
{
    constexpr int kMaxDevices = 64;
    static int cached[kMaxDevices]; // 0 = not looked up yet; a race between two first calls writes the same value
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return 256u;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        cached[dev] = n;
    }
    return (uint32_t)cached[dev];
}

} // namespace mxfp4

extern "C" {

mxfp4_status mxfp4_quant_from_fp8(const uint8_t *x, const float *x_scale, int64_t M_src, int64_t K,
                                  const int32_t *gather_idx, int64_t M_out, uint8_t *q, int64_t ld_q,
                                  uint8_t *sf, int64_t ld_sf, void *hip_stream)
{
    if (M_src < 0 || M_out < 0 || K < 0 || K % 128 != 0)
        return MXFP4_ERR_SHAPE;
    if (!gather_idx && M_out != M_src)
        return MXFP4_ERR_SHAPE;
    if (M_out == 0 || K == 0)
        return MXFP4_OK;
    if (!x || !x_scale || !q || !sf)
        return MXFP4_ERR_NULL;
    if (gather_idx && M_src == 0)
        return MXFP4_ERR_SHAPE;
    if (ld_q < K / 2 || ld_sf < K / 32 || M_src >= kMaxRows || M_out >= kMaxRows || K >= kMaxRows ||
        M_out * (K / 16) >= kMaxWorkItems)
        return MXFP4_ERR_SHAPE;
    if (!aligned(x, 16) || !aligned(x_scale, 4) || !aligned(q, 8) || ld_q % 8 != 0 || !aligned(sf, 4) ||
        ld_sf % 4 != 0 || (gather_idx && !aligned(gather_idx, 4)))
        return MXFP4_ERR_ALIGN;
    return launched(mxfp4::launch_quant_from_fp8(x, x_scale, M_src, K, gather_idx, M_out, q, ld_q, sf, ld_sf,
                                                 static_cast<hipStream_t>(hip_stream)));
}

mxfp4_status mxfp4_quant_from_fp8_scatter(const uint8_t *x, const float *x_scale, int64_t M_src, int64_t K,
                                          const int32_t *dst_idx, int32_t fanout, int64_t M_out, uint8_t *q,
                                          int64_t ld_q, uint8_t *sf, int64_t ld_sf, void *hip_stream)
{
    if (M_src < 0 || M_out < 0 || K < 0 || K % 128 != 0 || fanout <= 0)
        return MXFP4_ERR_SHAPE;
    if (M_src == 0 || M_out == 0 || K == 0)
        return MXFP4_OK;
    if (!x || !x_scale || !dst_idx || !q || !sf)
        return MXFP4_ERR_NULL;
    if (ld_q < K / 2 || ld_sf < K / 32 || M_src >= kMaxRows || M_out >= kMaxRows || K >= kMaxRows ||
        M_src * (K / 16) >= kMaxWorkItems)
        return MXFP4_ERR_SHAPE;
    if (!aligned(x, 16) || !aligned(x_scale, 4) || !aligned(q, 8) || ld_q % 8 != 0 || !aligned(sf, 4) ||
        ld_sf % 4 != 0 || !aligned(dst_idx, 4))
        return MXFP4_ERR_ALIGN;
    return launched(mxfp4::launch_quant_from_fp8_scatter(x, x_scale, M_src, K, dst_idx, fanout, M_out, q, ld_q, sf,
                                                         ld_sf, static_cast<hipStream_t>(hip_stream)));
}

mxfp4_status mxfp4_quant_from_bf16(const uint16_t *x, int64_t M, int64_t K, uint8_t *q, int64_t ld_q, uint8_t *sf,
                                   int64_t ld_sf, void *hip_stream)
{
    if (M < 0 || K < 0 || K % 128 != 0)
        return MXFP4_ERR_SHAPE;
    if (M == 0 || K == 0)
        return MXFP4_OK;
    if (!x || !q || !sf)
        return MXFP4_ERR_NULL;
    if (ld_q < K / 2 || ld_sf < K / 32 || M >= kMaxRows || K >= kMaxRows || M * (K / 8) >= kMaxWorkItems)
        return MXFP4_ERR_SHAPE;
    if (!aligned(x, 16) || !aligned(q, 4) || ld_q % 4 != 0 || !aligned(sf, 4) || ld_sf % 4 != 0)
        return MXFP4_ERR_ALIGN;
    return launched(mxfp4::launch_quant_from_bf16(x, M, K, q, ld_q, sf, ld_sf, static_cast<hipStream_t>(hip_stream)));
}

mxfp4_status mxfp4_dequant_to_fp8(const uint8_t *q, int64_t ld_q, const uint8_t *sf, int64_t ld_sf, int64_t M,
                                  int64_t K, uint8_t *x, float *x_scale, void *hip_stream)
{
    if (M < 0 || K < 0 || K % 128 != 0)
        return MXFP4_ERR_SHAPE;
    if (M == 0 || K == 0)
        return MXFP4_OK;
    if (!q || !sf || !x || !x_scale)
        return MXFP4_ERR_NULL;
    if (ld_q < K / 2 || ld_sf < K / 32 || M >= kMaxRows || K >= kMaxRows || M * (K / 16) >= kMaxWorkItems)
        return MXFP4_ERR_SHAPE;
    if (!aligned(q, 16) || ld_q % 16 != 0 || !aligned(x, 16) || !aligned(x_scale, 4))
        return MXFP4_ERR_ALIGN;
    return launched(mxfp4::launch_dequant_to_fp8(q, ld_q, sf, ld_sf, M, K, x, x_scale,
                                                 static_cast<hipStream_t>(hip_stream)));
}

static mxfp4_status row_to_col_common(const uint8_t *q_row, const uint8_t *sf_row, const int32_t *expert_offsets,
                                      int32_t num_experts, int64_t M, int64_t K, uint8_t *q_col,
                                      uint8_t *sf_col, void *hip_stream)
{
    // the flat form has whole column blocks; the splits of the grouped form may have any length
    if (M < 0 || K < 0 || K % 128 != 0 || (!expert_offsets && M % 32 != 0))
        return MXFP4_ERR_SHAPE;
    if (M == 0 || K == 0)
        return MXFP4_OK;
    if (!q_row || !sf_row || !q_col || !sf_col)
        return MXFP4_ERR_NULL;
    // byte offsets inside a 256-row tile are 32-bit, and so is the tile count
    if (M >= kMaxRows || K > ((int64_t)1 << 24) ||
        ((M + 255) / 256 + num_experts) * ((K + 255) / 256) >= ((int64_t)1 << 31))
        return MXFP4_ERR_SHAPE;
    if (!aligned(q_row, 4) || !aligned(sf_row, 4) || !aligned(q_col, 16) ||
        (expert_offsets && !aligned(expert_offsets, 4)))
        return MXFP4_ERR_ALIGN;
    return launched(mxfp4::launch_row_to_col(q_row, sf_row, expert_offsets, num_experts, M, K, q_col, sf_col,
                                             static_cast<hipStream_t>(hip_stream)));
}

mxfp4_status mxfp4_row_to_col(const uint8_t *q_row, const uint8_t *sf_row, int64_t M, int64_t K, uint8_t *q_col,
                              uint8_t *sf_col, void *hip_stream)
{
    return row_to_col_common(q_row, sf_row, nullptr, 0, M, K, q_col, sf_col, hip_stream);
}

mxfp4_status mxfp4_quant_from_fp8_grouped(const uint8_t *x, const float *x_scale, const int32_t *expert_offsets,
                                          int32_t num_experts, int64_t M_total, int64_t K, uint8_t *q,
                                          uint8_t *sf, void *hip_stream)
{
    if (num_experts <= 0 || num_experts > MXFP4_MAX_EXPERTS)
        return MXFP4_ERR_OFFSETS;
    if (!expert_offsets)
        return MXFP4_ERR_NULL;
    if (!aligned(expert_offsets, 4))
        return MXFP4_ERR_ALIGN;
    // rows are independent: the expert boundaries do not change any output byte
    return mxfp4_quant_from_fp8(x, x_scale, M_total, K, nullptr, M_total, q, K / 2, sf, K / 32, hip_stream);
}

mxfp4_status mxfp4_row_to_col_grouped(const uint8_t *q_row, const uint8_t *sf_row, const int32_t *expert_offsets,
                                      int32_t num_experts, int64_t M_total, int64_t K, uint8_t *q_col,
                                      uint8_t *sf_col, void *hip_stream)
{
    if (num_experts <= 0 || num_experts > MXFP4_MAX_EXPERTS)
        return MXFP4_ERR_OFFSETS;
    if (!expert_offsets)
        return MXFP4_ERR_NULL;
    return row_to_col_common(q_row, sf_row, expert_offsets, num_experts, M_total, K, q_col, sf_col, hip_stream);
}

static mxfp4_status row_to_fp8_col_common(const uint8_t *q_row, const uint8_t *sf_row,
                                          const int32_t *expert_offsets, int32_t num_experts, int64_t M,
                                          int64_t K, uint8_t *x_col, float *x_col_scale, void *hip_stream,
                                          bool requant = false)
{
    // the flat form has whole scale groups; the splits of the grouped form may have any length
    if (M < 0 || K < 0 || K % 128 != 0 || (!expert_offsets && M % 128 != 0))
        return MXFP4_ERR_SHAPE;
    if (M == 0 || K == 0)
        return MXFP4_OK;
    if (!q_row || !sf_row || !x_col || !x_col_scale)
        return MXFP4_ERR_NULL;
    // byte offsets inside a 256 x 256 tile are 32-bit on both sides, and so is the tile count
    if (M > ((int64_t)1 << 24) || K > ((int64_t)1 << 24) ||
        ((M + 255) / 256 + num_experts) * ((K + 255) / 256) >= ((int64_t)1 << 31))
        return MXFP4_ERR_SHAPE;
    if (!aligned(q_row, 4) || !aligned(sf_row, 4) || !aligned(x_col, 16) || !aligned(x_col_scale, 4) ||
        (expert_offsets && !aligned(expert_offsets, 4)))
        return MXFP4_ERR_ALIGN;
    const hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    return launched(requant ? mxfp4::launch_row_to_fp8_col_requant(q_row, sf_row, expert_offsets, num_experts, M, K,
                                                                   x_col, x_col_scale, stream)
                            : mxfp4::launch_row_to_fp8_col(q_row, sf_row, expert_offsets, num_experts, M, K, x_col,
                                                           x_col_scale, stream));
}

mxfp4_status mxfp4_row_to_fp8_col(const uint8_t *q_row, const uint8_t *sf_row, int64_t M, int64_t K,
                                  uint8_t *x_col, float *x_col_scale, void *hip_stream)
{
    return row_to_fp8_col_common(q_row, sf_row, nullptr, 0, M, K, x_col, x_col_scale, hip_stream);
}

mxfp4_status mxfp4_row_to_fp8_col_grouped(const uint8_t *q_row, const uint8_t *sf_row,
                                          const int32_t *expert_offsets, int32_t num_experts, int64_t M_total,
                                          int64_t K, uint8_t *x_col, float *x_col_scale, void *hip_stream)
{
    if (num_experts <= 0 || num_experts > MXFP4_MAX_EXPERTS)
        return MXFP4_ERR_OFFSETS;
    if (!expert_offsets)
        return MXFP4_ERR_NULL;
    return row_to_fp8_col_common(q_row, sf_row, expert_offsets, num_experts, M_total, K, x_col, x_col_scale,
                                 hip_stream);
}

mxfp4_status mxfp4_row_to_fp8_col_requant(const uint8_t *q_row, const uint8_t *sf_row, int64_t M, int64_t K,
                                          uint8_t *x_col, float *x_col_scale, void *hip_stream)
{
    return row_to_fp8_col_common(q_row, sf_row, nullptr, 0, M, K, x_col, x_col_scale, hip_stream, true);
}

mxfp4_status mxfp4_row_to_fp8_col_requant_grouped(const uint8_t *q_row, const uint8_t *sf_row,
                                                  const int32_t *expert_offsets, int32_t num_experts,
                                                  int64_t M_total, int64_t K, uint8_t *x_col, float *x_col_scale,
                                                  void *hip_stream)
{
    if (num_experts <= 0 || num_experts > MXFP4_MAX_EXPERTS)
        return MXFP4_ERR_OFFSETS;
    if (!expert_offsets)
        return MXFP4_ERR_NULL;
    return row_to_fp8_col_common(q_row, sf_row, expert_offsets, num_experts, M_total, K, x_col, x_col_scale,
                                 hip_stream, true);
}

mxfp4_status mxfp4_stream_copy(const void *src, void *dst, int64_t bytes, int32_t policy, void *hip_stream)
{
    return mxfp4_stream_mix(src, dst, bytes, policy, 0, hip_stream);
}

mxfp4_status mxfp4_stream_mix(const void *src, void *dst, int64_t bytes, int32_t policy, int32_t mix, void *hip_stream)
{
    if (bytes < 0 || bytes % 16 != 0 || policy < 0 || policy > 3 || mix < 0 || mix > 3 ||
        bytes / 16 / 512 >= ((int64_t)1 << 31))
        return MXFP4_ERR_SHAPE;
    if (bytes == 0)
        return MXFP4_OK;
    if (!src || !dst)
        return MXFP4_ERR_NULL;
    if (!aligned(src, 16) || !aligned(dst, 16))
        return MXFP4_ERR_ALIGN;
    return launched(mxfp4::launch_stream_copy(src, dst, bytes / 16, policy, mix, static_cast<hipStream_t>(hip_stream)));
}

mxfp4_status mxfp4_tile_copy(const void *src, void *dst, int64_t rows, int64_t row_bytes, void *hip_stream)
{
    if (rows < 0 || row_bytes < 0 || rows % 256 != 0 || row_bytes % 128 != 0 || rows >= kMaxRows ||
        row_bytes > ((int64_t)1 << 23) || (rows / 256) * (row_bytes / 128) >= ((int64_t)1 << 31))
        return MXFP4_ERR_SHAPE;
    if (rows == 0 || row_bytes == 0)
        return MXFP4_OK;
    if (!src || !dst)
        return MXFP4_ERR_NULL;
    if (!aligned(src, 16) || !aligned(dst, 16))
        return MXFP4_ERR_ALIGN;
    return launched(mxfp4::launch_tile_copy(src, dst, rows, row_bytes, static_cast<hipStream_t>(hip_stream)));
}

mxfp4_status mxfp4_record_fanout(const void *src, int64_t ld_src, const int32_t *dst_idx, int64_t M_src, int32_t fanout,
                                 int64_t rec_bytes, int64_t M_out, void *dst, void *hip_stream)
{
    if (M_src < 0 || M_out < 0 || fanout < 1 || rec_bytes <= 0 || rec_bytes % 16 != 0 || rec_bytes > 48 * 1024 ||
        ld_src < rec_bytes || M_src >= kMaxRows || M_out >= kMaxRows)
        return MXFP4_ERR_SHAPE;
    if (M_src == 0 || M_out == 0)
        return MXFP4_OK;
    if (!src || !dst || !dst_idx)
        return MXFP4_ERR_NULL;
    if (!aligned(src, 16) || !aligned(dst, 16) || ld_src % 16 != 0 || !aligned(dst_idx, 4))
        return MXFP4_ERR_ALIGN;
    return launched(mxfp4::launch_record_fanout(src, ld_src, dst_idx, M_src, fanout, rec_bytes, M_out, dst,
                                                static_cast<hipStream_t>(hip_stream)));
}

const char *mxfp4_status_string(mxfp4_status status)
{
    switch (status) {
    case MXFP4_OK: return "ok";
    case MXFP4_ERR_NULL: return "null pointer";
    case MXFP4_ERR_SHAPE: return "bad shape or stride";
    case MXFP4_ERR_ALIGN: return "misaligned pointer or stride";
    case MXFP4_ERR_OFFSETS: return "bad expert count";
    case MXFP4_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
    }
}

} // extern "C"
