"""MI355X-native hot path of R-TOSS pattern pruning: pattern selection, packing and
pattern-sparse convolution as hand-written HIP kernels behind a C ABI.

Importing the package does not load the GPU library; `paper_2303_02191_amd.binding`
loads it on first use and fails loudly if it has not been built.
"""
