"""MI355X-native decode-step hybrid-head sparse attention (LycheeDecode, Sec. 3.1 / Alg. 1).

`binding` wraps the C ABI of liblychee.so (include/lychee.h); `workloads` draws the seeded
synthetic inputs; `build` compiles the HIP sources.  Nothing here computes attention in
Python: every step of the path runs in the HIP kernels.
"""
