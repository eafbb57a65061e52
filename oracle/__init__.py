"""CPU oracle for the mixed-batch paged-attention path (TEST INFRASTRUCTURE ONLY).

Nothing in the product package imports this; only tests/, __graft_entry__.smoke()
and bench.py's cpu_baseline leg may use it.  It shares no code with the HIP path.
"""
