"""CPU oracle for the MemoSight decode hot path.  Test infrastructure only: imported by
tests, the smoke check and the benchmark's CPU-baseline leg, never by the product path."""
