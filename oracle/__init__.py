"""CPU oracle of the HeteroCache decode hot path: TEST INFRASTRUCTURE ONLY.

Plain fp64 C (hc_oracle.c) plus a thin ctypes loader and the per-step state machine
(ref.py).  Nothing in the product package may import this; only tests, the smoke check
and the benchmark's cpu_baseline leg do.
"""
