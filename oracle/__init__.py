"""CPU oracle of the PSB scalar-product layer: TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It shares no code with paper_1904_02205_amd.
"""
