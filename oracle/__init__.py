"""CPU oracle of the SGP update.  TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check
and the benchmark's CPU-baseline leg; never by the product package."""
