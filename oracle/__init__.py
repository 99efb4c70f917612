"""Plain CPU oracle of the aggregation + update path.  TEST INFRASTRUCTURE ONLY:
imported by tests, the smoke check and the benchmark's cpu_baseline leg, never by
the GPU library or its Python binding."""
