"""CPU oracles for the tuned-SGEMM path.  Test infrastructure only: the product package
never imports this; only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg do."""
