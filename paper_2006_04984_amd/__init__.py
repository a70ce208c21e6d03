"""Convolution with algorithm-based error detection for AMD gfx950.

Thin Python binding over libabed.so (see include/abed.h).  Importing this
package loads nothing; the library is opened on first use and a missing or
unbuilt library is an error (there is no fallback path)."""
from .binding import (ConvDesc, Layout, Variant, AbedError, lib, lib_path, get_layout, filter_prepare_int8,
                      input_checksum_int8, conv_int8, conv_int8_static, probe, workspace_init, desc_from_shape, filter_prepare_fp16,
                      input_checksum_fp16, conv_fp16, FicLayout, fic_get_layout, fic_filter_prepare_int8,
                      fic_input_checksum_int8, fic_conv_int8, ONLY_FC, ONLY_IC, PACKED_FC, LOCAL, L1_THRESHOLD, pad_channels, abft_gemm_get_layout, abft_gemm_int8, ABFT_TASKS, filter_prepare_local_int8, Ic2Layout, ic2_get_layout, ic2_conv_int8, fic_verify,
                      FicInloopLayout, FIC_INLOOP, fic_inloop_get_layout, fic_inloop_filter_prepare_int8, fic_inloop_conv_int8)

__all__ = ["ConvDesc", "Layout", "Variant", "AbedError", "lib", "lib_path", "get_layout", "filter_prepare_int8",
           "input_checksum_int8", "conv_int8", "conv_int8_static", "probe", "workspace_init", "desc_from_shape", "filter_prepare_fp16",
           "input_checksum_fp16", "conv_fp16", "FicLayout", "fic_get_layout", "fic_filter_prepare_int8",
           "fic_input_checksum_int8", "fic_conv_int8", "ONLY_FC", "ONLY_IC", "PACKED_FC", "LOCAL", "L1_THRESHOLD", "pad_channels", "abft_gemm_get_layout", "abft_gemm_int8", "ABFT_TASKS", "filter_prepare_local_int8", "Ic2Layout", "ic2_get_layout", "ic2_conv_int8", "fic_verify",
           "FicInloopLayout", "FIC_INLOOP", "fic_inloop_get_layout", "fic_inloop_filter_prepare_int8", "fic_inloop_conv_int8"]
