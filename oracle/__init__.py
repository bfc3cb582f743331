"""CPU oracle of the HDQT matmul path: test infrastructure only.

Imported by tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg.
The product package never imports this.
"""
