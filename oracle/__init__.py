"""CPU oracle for head-wise offloaded attention (HeadInfer, arXiv 2502.12574).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, fp64 restatement of what the GPU library must
compute.  Only the tests, the smoke check and the benchmark's CPU-baseline leg may import it; the product
path never does.  It shares no code with the GPU library and imports nothing from it.
"""
