"""CPU oracle (test infrastructure).  Only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may import this package; the product path never does."""
