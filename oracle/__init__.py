"""CPU oracle for the Breadcrumbs Reasoning decode / compress / masked-prefill path.

TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64 NumPy written from the paper
(arXiv 2510.13797).  It shares no code with the HIP library and imports
nothing from it; only the tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this package.  The product path never does.

Modules
-------
residency  which cache entries exist at every step of the generation loop
           (Alg. 1, Sec. 3.1) - literal list form, structured form, closed forms
attention  softmax attention over a given key set (Sec. 2: the standard
           Transformer attention), the training-time visibility rule (Fig. 2,
           Sec. 3.2) and the dense masked attention built from it
cache      a K/V-carrying cache simulator: append, beacon append, eviction
           (Alg. 1), with the same state/capacity error rules the library
           documents in its header

Pins (see tests/test_oracle_*.py): literal == structured == closed form,
brute force on tiny inputs, textbook/library attention as the no-eviction
special case, single-key / equal-key / scale-0 closed forms, permutation
invariance, GQA == MHA with repeated K/V, dominated-logit bound, mask
predicate == residency of the eviction loop, masked-prefill row == decode
over the evicted cache.  Numeric attention outputs have no printed example in
the paper: they are pinned by those identities, not by paper values.
"""
