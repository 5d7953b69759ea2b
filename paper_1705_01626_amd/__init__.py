"""Zero-value compression (ZVC) of sparse activation tensors on AMD MI355X.

`paper_1705_01626_amd.zvc` is a thin ctypes binding of the C ABI declared in
include/zvc.h (argument marshalling only; every step runs in the HIP kernels of
csrc/zvc.hip).  `paper_1705_01626_amd.workloads` draws the synthetic tensors
used by the tests and the benchmark.  The library is loaded on first use and
the import fails loudly there if it has not been built.
"""
