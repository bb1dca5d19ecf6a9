"""CPU oracle -- TEST INFRASTRUCTURE ONLY.

Plain, slow reference implementation of one data-parallel worker's SGD
iteration.  Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline
leg may import this package; the GPU product path never does.
"""
