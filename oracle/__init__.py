"""CPU oracle for the LiquidQuant W4A8 GEMM path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import, call or
link this directory: only tests/, __graft_entry__.smoke() and the cpu_baseline
leg of bench.py use it.  It shares no code with the HIP path.
"""
