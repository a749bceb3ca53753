"""CPU oracle for the forest-verification path of dynamic-width speculative beam decoding.

TEST INFRASTRUCTURE ONLY.  Plain, slow numpy fp64 code written from the paper so
that it can be checked against the paper by eye.  Only the tests, the smoke check
and the benchmark's `cpu_baseline` leg may import it; the product path (the HIP
library and its Python binding) never does, and shares no code with it.

Parity pins (tests/test_oracle_*.py):
  forest topology ........ pinned (boolean-matrix transitive closure)
  forest attention ....... pinned (library causal / masked attention, GQA and shared-prefix invariances)
  log-softmax ............ pinned (scipy / torch library routines)
  accept / residual ...... pinned (standard speculative sampling at W=1; appendix identities;
                           exhaustive enumeration of Theorem 3.1 on tiny vocabularies)
  dynamic width .......... pinned (Eq. 1-2 invariants; exact accept-count distribution by enumeration)
  inverse-CDF sampling convention, role-indexed uniforms, tie-breaks:
                           parity unpinned by the paper (conventions of this build), checked by
                           brute force on tiny inputs and a frequency test only.
"""
