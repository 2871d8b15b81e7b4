"""CPU oracle for the DyBit quantize + GEMM/conv path.

TEST INFRASTRUCTURE ONLY.  Slow, plain and written from the paper's definitions
(Sec. III-A, Eq. 1, Table I, and the decoder/encoder description in Sec. III-B).
It shares no code with the HIP library and must never be imported by the
product path: only tests, the smoke check and the benchmark's cpu_baseline leg
may use it.
"""
