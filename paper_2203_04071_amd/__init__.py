"""MI355X-native table-lookup GEMM / convolution for approximate-multiplier emulation
(hot path of AdaPT, arXiv 2203.04071).

Sub-modules: `binding` (ctypes wrapper of the C ABI in include/adapt_mi355.h), `networks`
(CNN / LSTM / GAN workloads as sequences of ABI calls), `workloads` (seeded synthetic inputs,
no arithmetic of the method), `build` (hipcc build of csrc/).  Nothing is imported eagerly so that
`workloads` can be used without the HIP library.
"""
