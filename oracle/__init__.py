"""CPU oracle for the coalesced-superkernel path -- TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 definitions of what every operator in a superkernel must
compute (Sections 1 and 5.3: coalescing packs independent GEMM-backed
operators into one launch without changing their results), the storage-type
rounding helpers, the reference tile planner and its coverage checker, and
the error measures the parity tests gate on.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It imports nothing from the product package and shares no code
with the HIP path.
"""
