"""CPU oracle and brute-force checkers: test infrastructure only.

Nothing in the product path (paper_2605_00342_amd) imports this package; it is used by
tests/, __graft_entry__.smoke() and the cpu_baseline leg of bench.py.
"""
