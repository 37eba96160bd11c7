"""Slow fp64 CPU oracle (numpy).  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package; the product package never does and shares no code with it.
"""
