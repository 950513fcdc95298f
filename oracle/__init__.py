"""CPU oracle for the LazyTensor fused-execution path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this
directory; only tests/, __graft_entry__.smoke() and the cpu_baseline leg of
bench.py do.  It shares no code with the HIP/C++ library.

Two independent parts:

* ``oracle.numeric``    -- an op-by-op eager evaluator: every tensor op is run
  the moment it is issued and every intermediate is materialised.  That is
  the plain definition of what a lazily traced and fused program must equal
  (section 3 of the paper: compiled traces are semantically equivalent to
  running the operations one at a time).
* ``oracle.structural`` -- a second, independent implementation of the trace
  recorder, canonical numbering, serialisation, hash, 0/1 folding and region
  partitioner, written from the same written specification as the C++ library.

Parity status: every function here is pinned by tests that run without a GPU
(tests/test_oracle_*.py): closed forms, brute force in float64, the IR
listings printed in the paper's figures 1-3, published FNV-1a vectors and
structural invariants.  Nothing is "parity unpinned".
"""
