"""CPU oracle for the GAS layer step.  TEST INFRASTRUCTURE, not product code:
only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may use
it.  It shares no code with the HIP library and never imports it."""
