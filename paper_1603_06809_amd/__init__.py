"""Virtual-rank MPI broadcast (binomial scatter + ring allgather, native and
tuned) executed on one GPU.  ``inputs`` holds the seeded workloads; ``vbcast``
is the thin binding over the C-ABI library built from ``csrc/``."""
