"""CPU oracles for the Stream-K++ hot path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this
directory; only the tests, the smoke check and the benchmark's CPU-baseline
leg may call it.  Everything here is deliberately slow and written straight
from the definitions so that it can be checked against the paper by eye.

Modules
-------
schedule   integer scheduler: iteration-to-workgroup mapping for the seven
           policies (Algorithm 1, Sec. 3.2, Sec. 4.1)
simulate   executes a schedule segment by segment with fp32 partial tiles and a
           fixed-order fix-up (Sec. 5.3's "parallel reduction" alternative)
bloom      Murmur3-keyed Bloom filters, one per policy (Sec. 4.2)
gemm       triple-loop GEMM with fp64 accumulation (Sec. 1, "GEMM"), C + ctypes
"""
