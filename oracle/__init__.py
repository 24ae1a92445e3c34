"""CPU oracle of the CARD verify step and shared cache.  TEST INFRASTRUCTURE ONLY:
only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import it."""
