"""Float64 CPU oracle of the fused chain.  TEST INFRASTRUCTURE: imported only by tests/,
the smoke check and the benchmark's CPU-baseline leg; never by the product package."""
