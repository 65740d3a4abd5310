"""CPU oracle of the Cool-SD verify-and-resample stage.

TEST INFRASTRUCTURE: only tests/, __graft_entry__.smoke() and the cpu_baseline
leg of bench.py may import this package.  It shares nothing with the HIP library.
"""
