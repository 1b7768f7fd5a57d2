"""CPU oracle of the approximate-gradient-coding hot path: test infrastructure only.

Nothing in the product package imports this; only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py do.
"""
