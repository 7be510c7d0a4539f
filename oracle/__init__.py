"""CPU oracle for the AMS-KV hot path.  Test infrastructure only: imported by the tests,
by the smoke check and by the benchmark's CPU-baseline leg, never by the product path."""
