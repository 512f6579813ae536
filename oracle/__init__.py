"""CPU oracle for the per-token core of Truncated PPO (T-PPO).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library and
its Python binding) imports, links or calls anything in this package; only the
test-suite, the smoke check and the CPU-baseline leg of the benchmark do.
The oracle shares no code with the HIP path.

Two levels, both written from the paper's definitions:

* ``oracle.definitional`` -- pure-Python fp64 loops that evaluate each
  equation exactly as printed (explicit sums, ``math.fsum``); O(T^2) where the
  equation is a sum.  Used on tiny inputs to pin the level below.
* ``oracle.fast`` -- numpy fp64: the backward recurrences that the sums
  telescope into, and a BLAS matrix product followed by the textbook
  log-softmax for the LM head.  This is what the GPU results are compared to.

Parity status: every function in both modules is pinned by the CPU tests
(closed forms, special cases, hand-worked examples, brute force); none is
"parity unpinned".
"""
