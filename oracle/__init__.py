"""CPU oracle for the EoRA compensated compressed linear layer (arXiv 2410.21271).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, float64 numpy
implementation of what the GPU hot path computes:

    y = x . What^T + (x . A^T) . B^T            (Sec. 3, forward equation; Alg. 1 step 7)

with What either a group-wise 3/4-bit quantised weight (asymmetric: scale and
integer zero-point per group, Sec. 4.1 / App. A.11) or a 2:4 structured-sparse
fp16 weight (Sec. 1, Sec. 4.2), and A, B the rank-r EoRA factors in fp16 or
4-bit (Sec. 4.5, "quantised EoRA").

It shares no code with the HIP library: it neither imports the product package
nor is imported by it.  Only the tests, the smoke check and the bench's
`cpu_baseline` leg may call it.

Modules
-------
layout     bit-level pack / unpack of every stored format (integer work)
linear     dequantisation, 2:4 expansion and the float64 forward pass
calibrate  Algorithm 1 steps 1-6 (offline eigenspace projection), used only to
           build realistic factors and to pin the forward pass on planted errors

Parity status: every function here is pinned by tests/test_oracle_*.py (hand
computed bit patterns under tests/golden/, exact-rational brute force, planted
rank-r reconstruction, closed forms of Theorem 1).  No function is "parity
unpinned".
"""
