"""MI355X-native single-GPU k-NN-graph construction (lock-free NN-Descent).

`workloads` (input generators) imports without the GPU library; everything
else lives in `knng` (the ctypes binding over libknng.so) and is imported on
first use so that a missing library fails loudly at the call site.
"""
__all__ = ["workloads", "knng"]
