"""fp64 CPU checker for the device library.  TEST INFRASTRUCTURE ONLY: imported
by tests/, the smoke check and the benchmark's CPU-baseline leg; never by the
product path.  Shares no code with the HIP sources."""
