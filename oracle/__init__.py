"""CPU oracle for the KV-CAR decode hot path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this
directory; it is used by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py.  It shares no code with the HIP path.
"""
