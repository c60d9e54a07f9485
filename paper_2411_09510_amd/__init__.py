"""mxc — block-quantized communication compression for tensor-parallel partial activations,
MI355X (gfx950).  Thin Python binding over the C-ABI library ``libmxc.so``; every step of the
path runs in the library's HIP kernels, PyTorch only provides device memory and streams."""
from .binding import (Format, Launch, MxcError, copy_probe, dequant_reduce,
                      dequant_reduce_own, dequant_reduce_requantize, effective_bits, int_format,
                      lib,
                      prepare_dequant_reduce_requantize,
                      packed_sizes, prepare_dequant_reduce, prepare_quantize_batched,
                      prepare_requantize_chunk, quantize, quantize_batched, requantize_chunk,
                      time_next_launch, version)

__all__ = ["Format", "Launch", "MxcError", "copy_probe", "dequant_reduce",
           "dequant_reduce_own", "dequant_reduce_requantize", "prepare_dequant_reduce_requantize",
           "int_format", "effective_bits", "lib",
           "packed_sizes", "prepare_dequant_reduce", "prepare_quantize_batched",
           "prepare_requantize_chunk", "quantize", "quantize_batched", "requantize_chunk",
           "time_next_launch", "version"]
