"""CPU oracle of the Swimba token mixer.  TEST INFRASTRUCTURE ONLY: imported by
the tests, the smoke check and the benchmark's cpu_baseline leg, never by the
product path."""
