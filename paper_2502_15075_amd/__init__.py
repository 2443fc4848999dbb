"""kvq: key-prioritized mixed-precision KV cache (quantize-append, dequantize, decode attention) for MI355X."""
