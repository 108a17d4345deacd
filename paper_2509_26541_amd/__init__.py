"""One rank's share of TASP (topology-aware sequence parallelism) on one MI355X.

The work is done by a C-ABI library of HIP kernels (csrc/, include/tasp.h); `binding` marshals
arguments to it and nothing else.  Importing this package does not load the library; `binding`
does, and fails loudly when it has not been built.
"""
