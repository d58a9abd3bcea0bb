"""CPU oracle for the HE-based federated aggregation hot path (FedML-HE, Algorithm 1).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, step-by-step CPU
implementation (numpy uint64 / float64 and Python big integers) of what the
GPU library computes.  It shares no code, tables or constants with the HIP
path and must never be imported by the product package.  Only the tests, the
smoke check and the benchmark's CPU-baseline leg may call it.

What the paper fixes and what it does not
-----------------------------------------
The paper fixes *what* is aggregated: the server forms
    [W_glob] = sum_i alpha_i [[M . W_i]] + sum_i alpha_i ((1-M) . W_i)
(Section "Algorithm for HE-Based Federated Aggregation", Algorithm 1), with
plaintext weights alpha_i and one multiplicative depth, on the CKKS scheme
(Section "Homomorphic Encryption") with a packing batch per ciphertext
(Section "Default Crypto Parameters").  It treats the HE scheme itself as a
library call and prints no ring-level value anywhere, so every ring-level
step below follows the textbook RNS-CKKS construction with the parameter
choices named in each module's header.

Parity pins
-----------
Every function is pinned by tests that do not re-type its formula: brute
force on tiny rings, closed forms, algebraic invariants and published
known-answer vectors (see tests/test_oracle_*.py).  One thing stays
"parity unpinned": the actual bytes of a ciphertext or key, because the paper
prints none; those are compared GPU <-> oracle only, after every operation
that produces them has been pinned by the invariants above.
"""
