"""MI355X-native FastSGD gradient codec (arXiv 2112.04291, Section 3): HIP kernels behind a C ABI.

`paper_2112_04291_amd.binding` is the thin ctypes layer over the C-ABI library; importing this
package does not load the library (the input generators in `workloads` have no GPU dependency).
"""
__all__ = ["binding", "workloads", "build"]
