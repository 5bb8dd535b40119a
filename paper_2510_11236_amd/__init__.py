"""MI355X-native quantized-KV decode attention (XQuant hot path) -- Python binding of libxq."""
from .binding import (XQ_DECODE_MATRIX_F16, XQ_DECODE_MERGE_IN_LAUNCH, XQ_DECODE_MERGE_LAUNCH, XQ_DECODE_PAIR_FUSED, XQ_DECODE_VECTOR_ALU, XqCache, XqConfig, XqError, cache_bytes, equivalent_bits, lib,
                      strerror)

__all__ = ["XqConfig", "XqCache", "XqError", "cache_bytes", "equivalent_bits", "lib", "strerror",
           "XQ_DECODE_PAIR_FUSED", "XQ_DECODE_VECTOR_ALU", "XQ_DECODE_MATRIX_F16", "XQ_DECODE_MERGE_LAUNCH", "XQ_DECODE_MERGE_IN_LAUNCH"]
