"""MI355X-native GR forward (FLAME's fused-kernel hot path) behind a C-ABI library.

`workloads` (numpy only) is always importable; the binding to the HIP library is loaded lazily
by `paper_2509_22681_amd.binding` and raises if the library has not been built.
"""
