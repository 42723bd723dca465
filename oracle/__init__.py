"""CPU oracles for the KLA hot path: TEST INFRASTRUCTURE ONLY.

token_oracle  - fp64 token-by-token recurrence (plain C, Algorithm 1 left panel) and its gradient by
                reverse accumulation through the same lines
chunk_oracle  - fp64 numpy chunkwise solver (Algorithm 1 right panel, eqs. (6)-(8)), its gradient, and
                the diagonal-gating variant of App. B

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It never imports the GPU package and the GPU package never
imports it.  Every function is pinned in tests/test_oracle_pins.py; none is
"parity unpinned".
"""
