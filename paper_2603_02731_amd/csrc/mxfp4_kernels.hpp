// Launchers of the gfx950 kernels (internal to the library; the public boundary is the C
// ABI in include/mxfp4.h).  Arguments are already validated by the caller.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mxfp4 {

hipError_t launch_quant_from_fp8(const uint8_t *x, const float *x_scale, int64_t M_src, int64_t K,
                                 const int32_t *gather_idx, int64_t M_out, uint8_t *q, int64_t ld_q,
                                 uint8_t *sf, int64_t ld_sf, hipStream_t stream);

// Source row i goes to the output rows dst_idx[i*fanout .. i*fanout + fanout - 1].
hipError_t launch_quant_from_fp8_scatter(const uint8_t *x, const float *x_scale, int64_t M_src, int64_t K,
                                         const int32_t *dst_idx, int32_t fanout, int64_t M_out, uint8_t *q,
                                         int64_t ld_q, uint8_t *sf, int64_t ld_sf, hipStream_t stream);

hipError_t launch_quant_from_bf16(const uint16_t *x, int64_t M, int64_t K, uint8_t *q, int64_t ld_q, uint8_t *sf,
                                  int64_t ld_sf, hipStream_t stream);

hipError_t launch_dequant_to_fp8(const uint8_t *q, int64_t ld_q, const uint8_t *sf, int64_t ld_sf,
                                 int64_t M, int64_t K, uint8_t *x, float *x_scale, hipStream_t stream);

// expert_offsets == nullptr: the flat conversion of an [M, K] matrix.
hipError_t launch_row_to_col(const uint8_t *q_row, const uint8_t *sf_row, const int32_t *expert_offsets,
                             int32_t num_experts, int64_t M, int64_t K, uint8_t *q_col, uint8_t *sf_col,
                             hipStream_t stream);

// expert_offsets == nullptr: the flat conversion of an [M, K] matrix.
hipError_t launch_row_to_fp8_col(const uint8_t *q_row, const uint8_t *sf_row, const int32_t *expert_offsets,
                                 int32_t num_experts, int64_t M, int64_t K, uint8_t *x_col, float *x_col_scale,
                                 hipStream_t stream);

// The same conversion under the re-quantization reading (scale from the group maximum).
hipError_t launch_row_to_fp8_col_requant(const uint8_t *q_row, const uint8_t *sf_row, const int32_t *expert_offsets,
                                         int32_t num_experts, int64_t M, int64_t K, uint8_t *x_col,
                                         float *x_col_scale, hipStream_t stream);

// Compute units of the current device (hipDeviceAttributeMultiprocessorCount, looked up once per device;
// 256 if the runtime cannot say): launch heuristics are stated in tiles per compute unit.
uint32_t compute_units();

// Byte movers without arithmetic (the measured roofs).  `chunks` = work items of the stream mover (16 bytes of
// the wider side each); policy bit 0 = non-temporal loads, bit 1 = non-temporal stores; mix 0 = 1:1 copy,
// 1 = 2:1 (16 bytes read, 8 written), 2 = 1:2 (8 read, 16 written), 3 = read only.
hipError_t launch_stream_copy(const void *src, void *dst, int64_t chunks, int32_t policy, int32_t mix,
                              hipStream_t stream);
// A [rows, row_bytes] byte matrix moved tile by tile into the [2 * row_bytes, rows / 2] layout.
hipError_t launch_tile_copy(const void *src, void *dst, int64_t rows, int64_t row_bytes, hipStream_t stream);
// Record i of src (rec_bytes at src + i * ld_src) written to the records dst_idx[i * fanout + j] of dst.
hipError_t launch_record_fanout(const void *src, int64_t ld_src, const int32_t *dst_idx, int64_t M_src, int32_t fanout,
                                int64_t rec_bytes, int64_t M_out, void *dst, hipStream_t stream);

} // namespace mxfp4
