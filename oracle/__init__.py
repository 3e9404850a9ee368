"""CPU oracle for the PipeMax stage-decode hot path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this
directory; only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline
leg may use it.  It shares no code with the HIP path.
"""
