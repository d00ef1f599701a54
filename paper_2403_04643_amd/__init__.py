"""MI355X-native quality-adaptive KV-cache quantization (QAQ, arXiv 2403.04643).

The compute path lives in the C-ABI library built from csrc/ (hand-written HIP
for gfx950); `paper_2403_04643_amd.qaq` is the thin ctypes binding over it.
Importing this package does not load the library; `qaq.load()` does, and it
raises if the library has not been built.
"""
__all__ = ["qaq", "workloads"]
