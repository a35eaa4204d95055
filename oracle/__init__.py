"""CPU oracle for the Endor bitmap sparse format.  TEST INFRASTRUCTURE ONLY:
imported by tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg, never
by the product package."""
