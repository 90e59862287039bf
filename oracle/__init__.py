"""CPU oracle (test infrastructure only).

Plain, slow, fp64 numpy implementation of what the padding-free encoder path
must compute, written from the paper's definitions on *padded* tensors.
Nothing in the product path may import this package: only the tests, the
smoke check and the bench's cpu_baseline leg use it.
"""
