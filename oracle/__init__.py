"""CPU oracle for the Dynamic SplitFuse attention step (TEST INFRASTRUCTURE).

This package is the slow, plain definition the HIP library is checked against.
It is test infrastructure, not product code: only tests, the smoke check and the
benchmark's cpu_baseline leg may import it.  It shares no code with the HIP path
and never imports it.

Contents
--------
attention.py  blocked (paged) KV cache append + dense per-sequence causal softmax
              attention in fp64 (paper Sec. 2 "two phases", Sec. 2.1 blocked KV cache,
              Sec. 3.2 chunks of a prompt across forward passes).
composer.py   reference Dynamic SplitFuse batch composer with a block allocator
              (paper Sec. 2.2 continuous batching, Sec. 3.2 rules 1 and 2).

Pinning status
--------------
Every function is pinned by mathematical checks in tests/test_oracle_*.py (brute
force on tiny inputs, closed forms, chunking invariance, block-permutation
invariance, a library fp64 causal attention for the uncached case, composer
invariants).  The paper prints no worked numeric example for this path, so the
absolute output values for random inputs are pinned only through those checks.
"""
