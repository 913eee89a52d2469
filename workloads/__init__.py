"""Seeded synthetic inputs for the MADDNESS hot path.

This module only draws numbers: it holds none of the method's arithmetic (no
hashing, no tables, no scan) and is the one piece of code that both the CPU
oracle's tests and the HIP path's tests/bench may share.  Every array is
produced once, on the host, and the same bytes are handed to both sides.

The five workloads stand in for the paper's experiments, whose data sets are
not available here: workloads 1-2 take the shapes of the CIFAR-10/100 softmax
experiment (Section 5.3: A 10000x512, B 512x10 / 512x100), workload 3 takes the
structure of the image-filter experiment (Section 5.5 and Appendix E.6: 3x3
windows of an RGB image in CHW order, Sobel and Gaussian filters, two columns
of B), workloads 4-5 scale workload 2 up to throughput sizes.
"""
from .generators import (  # noqa: F401
    CHUNK,
    Workload,
    WORKLOADS,
    get_workload,
    make_B,
    make_A_train,
    make_A_chunk,
    make_A,
    n_chunks,
    chunk_rows,
    random_problem,
)
