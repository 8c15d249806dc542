"""CPU oracle for the TACO compression operator.  Test infrastructure only:
importable from tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg."""
