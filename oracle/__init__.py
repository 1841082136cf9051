"""Float64 CPU oracle for the HessFormer hot path (HVP + Lanczos + SLQ read-out).

TEST INFRASTRUCTURE ONLY.  This package is a slow, plain restatement of what
the paper's Algorithm 1 (Hessian-vector product) and Algorithm 2 (Lanczos)
compute, used to check the HIP implementation.  It shares no code with the HIP
path and must never be imported by it; only tests/, the smoke check and the
CPU-baseline leg of the benchmark use it.
"""
