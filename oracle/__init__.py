"""CPU oracle for tree attention: TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 implementations (numpy; the per-key gradient oracle uses plain
torch ops, on the CPU unless a test asks for another device) of what the tree-attention hot path
computes, written from the paper's statement of the problem.  Only the tests,
the smoke check and the benchmark's cpu_baseline leg may import this package;
the product path never does, and this package never imports the HIP binding.
"""
