"""MI355X-native FP8 <-> software-MXFP4 conversions (gfx950 HIP kernels behind a C ABI).

The Python layer only marshals arguments; see include/mxfp4.h for the boundary.
"""
from .binding import (Mxfp4Error, lib, mxfp4_dequant_to_fp8, mxfp4_quant_from_bf16, mxfp4_quant_from_fp8,
                      mxfp4_quant_from_fp8_grouped, mxfp4_quant_from_fp8_scatter, mxfp4_row_to_col, mxfp4_row_to_col_grouped,
                      mxfp4_row_to_fp8_col, mxfp4_row_to_fp8_col_grouped, mxfp4_stream_copy, mxfp4_stream_mix, mxfp4_tile_copy, mxfp4_record_fanout, status_string)

__all__ = ["Mxfp4Error", "lib", "mxfp4_dequant_to_fp8", "mxfp4_quant_from_bf16", "mxfp4_quant_from_fp8",
           "mxfp4_quant_from_fp8_grouped", "mxfp4_quant_from_fp8_scatter", "mxfp4_row_to_col", "mxfp4_row_to_col_grouped", "mxfp4_row_to_fp8_col",
           "mxfp4_row_to_fp8_col_grouped", "mxfp4_stream_copy", "mxfp4_stream_mix", "mxfp4_tile_copy", "mxfp4_record_fanout", "status_string"]
