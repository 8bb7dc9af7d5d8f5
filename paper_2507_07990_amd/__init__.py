"""MI355X-native spatio-temporal token merging (STTM): HIP library + thin ctypes binding.

`binding` loads the in-tree libsttm.so (built by `build`); `workloads` draws the seeded synthetic inputs.
"""
__all__ = ["binding", "build", "workloads"]
