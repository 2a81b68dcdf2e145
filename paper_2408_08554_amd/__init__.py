"""MI355X-native arbitrary-precision quantized matmul (ABQ-LLM hot path).

The compute lives in csrc/ (hand-written HIP for gfx950 behind a C ABI, include/abq.h);
`binding` marshals torch tensors into that ABI and nothing else.  The library is loaded on
first use and a missing build is an error, never a fallback.
"""
__all__ = ["binding", "synth"]
