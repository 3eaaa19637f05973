"""CPU oracle for the speculative-round hot path (test infrastructure, not product).

A plain float64 numpy implementation of what the HIP library computes, written
from the paper's definitions (Alg. 1 of the supplement, Eq. 1, Sec. 4.3, S2.1, S3)
and, where the paper is silent (transformer and head internals, KV cache), from
the readings listed in the design document.  It shares no code with the HIP path
and must not import it; only the tests, the smoke check and the benchmark's
`cpu_baseline` leg may import this package.

Pinned by tests/test_oracle_*.py against closed forms, invariants and brute-force
loops (oracle/loops.py).  End-to-end numerical values at the large configurations
have no external reference: parity there is pinned by those invariants only.
"""
