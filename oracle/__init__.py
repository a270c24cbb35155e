"""CPU oracle of the head-shard attention path.  Test infrastructure only: imported by
tests, the smoke check and the benchmark's CPU-baseline leg, never by the product path."""
