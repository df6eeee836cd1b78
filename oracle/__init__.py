"""CPU oracle: a plain, slow, independent implementation of what the GPU path computes.

TEST INFRASTRUCTURE ONLY.  Only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may import this package.  It shares no code with
paper_2203_15980_amd and neither imports the other.
"""
