"""MI355X-native implementation of the TACO fused FP8 compression operator
(block partition, Adaptive Scale-Hadamard transform, Dual-Scale FP8 quantisation and the
fused inverse).  The compute lives in a C-ABI HIP library (csrc/, include/taco.h);
`taco` is the thin ctypes binding and `workloads` the synthetic input generators."""

__all__ = ["taco", "workloads"]
