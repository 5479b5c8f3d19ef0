"""CPU oracle for the KVzap prune step.

TEST INFRASTRUCTURE ONLY. Nothing under this package is part of the product
path: it may be imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py, and by nothing else.  It shares no code with the
HIP library and never imports it.
"""
