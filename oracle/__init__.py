"""ORACLE -- test infrastructure only.

Plain, slow CPU implementations of what the ChunkFlow hot path computes, written from the paper:
  oracle.chunking   chunk construction (Algorithm 1) and state-aware scheduling (Algorithm 2),
                    plain Python integers
  oracle.attention  fp64 causal attention forward/backward, both as the textbook definition on
                    whole sequences and as the chunked method with retained key/value state
                    (ctypes wrapper over oracle/attention.c)

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this package.
It imports nothing from the HIP path and the HIP path imports nothing from it.
"""
