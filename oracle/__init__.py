"""CPU oracle for the LSR LM head.  TEST INFRASTRUCTURE ONLY.

Nothing under this package is part of the product path: only tests/, the smoke check in
__graft_entry__ and bench.py's cpu_baseline leg may import it.  It shares no code with the
HIP library and never imports it.
"""
