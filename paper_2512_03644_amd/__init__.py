"""MI355X-native snapshot pack / CRC32C / restore and fused AdamW snapshot.

The work is done by hand-written HIP kernels behind a C ABI (include/ffsnap.h); `binding`
marshals arguments for it, `workloads` draws the seeded synthetic inputs.  Importing the package
loads nothing heavy; the shared library is opened on first use and its absence is an error.
"""
__all__ = ["binding", "workloads"]
