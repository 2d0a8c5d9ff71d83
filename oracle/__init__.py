"""CPU oracle (test infrastructure only).

Plain fp64 statements of what the GPU library computes, written from the paper:
shared-KV attention (Sec. 3.2), the layer-dissimilarity matrix (Sec. 3.1.2) and the
structural part of the strategy search (Algorithm 1).  Nothing in the product path may
import this package; the tests, the smoke check and the benchmark's CPU-baseline leg do.
"""
