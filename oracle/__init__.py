"""fp64 CPU oracle for the DASH hot path. Test infrastructure, not product code.

Only tests, the smoke check and the CPU-baseline leg of the benchmark import this.
"""
