"""MI355X-native tree verify for budget-aware tree speculative decoding.

`synth`   seeded synthetic inputs (numpy only, no method arithmetic)
`binding` ctypes face of libbastion_tv.so (needs torch for device buffers; imported on demand)
`build`   hipcc build of the shared library
"""
__all__ = ["synth", "binding", "build"]
