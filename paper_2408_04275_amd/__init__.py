"""MI355X-native forward/backward of one transformer layer over a packed multimodal microbatch.

`workloads` draws seeded synthetic inputs; `binding` is the thin ctypes layer over
the C-ABI library built from `csrc/` (imported lazily: the library needs a GPU).
"""
__all__ = ["workloads", "binding", "parity"]
