"""MI355X-native head-wise paged KV-cache attention for colocated multi-LLM serving.

The GPU library (HIP kernels behind a C ABI, see include/mux.h) is loaded lazily by
`paper_2404_02015_amd.binding`; importing the package alone touches no GPU code, so the
seeded input generators in `paper_2404_02015_amd.workloads` can be used anywhere.
"""
__all__ = ["binding", "workloads", "build"]
