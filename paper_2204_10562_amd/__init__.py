"""MI355X-native batched evaluation of synchronous-pipeline plans (arXiv 2204.10562).

`binding` wraps the C ABI of libpp.so (include/pp.h); `workloads` holds the seeded
synthetic inputs; `build` compiles the HIP sources.
"""
