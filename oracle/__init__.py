"""CPU oracle (test infrastructure).  See ms_oracle.c for what it computes.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may
import this package; the product package never does.
"""
