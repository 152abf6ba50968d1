"""CPU oracle for tree attention: TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 numpy implementations of what the tree-attention hot path
computes, written from the paper's statement of the problem.  Only the tests,
the smoke check and the benchmark's cpu_baseline leg may import this package;
the product path never does, and this package never imports the HIP binding.
"""
