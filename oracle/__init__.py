"""CPU oracle of the FP8 <-> MXFP4 conversions (test infrastructure only).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this.
"""
