"""MI355X-native baseline-JPEG decoder built around self-synchronising parallel Huffman decoding
(Weissenberger & Schmidt, "Accelerating JPEG Decompression on GPUs", arXiv 2111.09219).

The package is a thin binding over the C ABI of include/jpgd.h; all decoding runs in the gfx950
kernels of csrc/.  Names follow the header.
"""
from .binding import (Batch, Config, F_NO_PIXELS, F_PLANAR, F_SCALE_2, F_SCALE_4, F_SCALE_8, STATIC_WORKSPACE_BYTES, KERNELS,
                      jpgd_decode_batch_async, jpgd_wait, jpgd_init, jpgd_static_workspace_bytes, jpgd_decode_static,
                      scale_denominator, Info, JpgdError, Report, EXPORTS, jpgd_decode, jpgd_decode_batch,
                      jpgd_parse, jpgd_read_sync_info, jpgd_unstuff, jpgd_workspace_bytes, library_path,
                      prepare_batch)
from .build import build

__all__ = ["Batch", "Config", "F_NO_PIXELS", "F_PLANAR", "F_SCALE_2", "F_SCALE_4", "F_SCALE_8", "STATIC_WORKSPACE_BYTES",
           "jpgd_decode_batch_async", "jpgd_wait", "jpgd_init", "jpgd_static_workspace_bytes", "jpgd_decode_static",
           "scale_denominator", "KERNELS", "Info", "JpgdError", "Report", "EXPORTS", "jpgd_decode",
           "jpgd_decode_batch", "jpgd_parse", "jpgd_read_sync_info", "jpgd_unstuff", "jpgd_workspace_bytes",
           "library_path", "prepare_batch", "build"]
