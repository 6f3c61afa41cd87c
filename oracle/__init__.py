"""CPU oracle (test infrastructure only).  Not part of the product path: only tests/,
__graft_entry__.smoke() and bench.py's cpu_baseline leg may import this package."""
