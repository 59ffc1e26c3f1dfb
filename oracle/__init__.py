"""CPU fp64 oracle.  TEST INFRASTRUCTURE: imported only by tests, the smoke check and the
benchmark's cpu_baseline leg; never by the product path."""
