"""CPU oracle of the paged KV-cache swap.  TEST INFRASTRUCTURE ONLY: imported by
tests/, the smoke check and the benchmark's CPU-baseline leg, never by the
product path."""
