"""CPU oracle for multimodal-masked attention under workload-balanced context
parallelism (paper section 3.2 "Token Workload-Balanced Context Parallelism",
section 4.2 "Implementation of MLLM Attention", Alg. 1).

TEST INFRASTRUCTURE ONLY.  Plain, slow, float64 / exact-integer code written
from the definitions; it shares nothing with the HIP path and must never be
imported by the product package.  Only tests, the smoke check and the
benchmark's cpu_baseline leg may use it.

Parity pins (what each function is checked against, other than itself) are
listed at the top of each module; the paper's timing tables are
"parity unpinned" (other hardware, unstated precision and CP degree).
"""
