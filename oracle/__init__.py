"""fp64 CPU oracle for packed varlen causal attention.  TEST INFRASTRUCTURE ONLY: imported by
tests/, by __graft_entry__.smoke() and by bench.py's cpu_baseline leg, never by the product."""
