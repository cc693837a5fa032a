"""CPU oracle of the failure-remapped MoE layer.  Test infrastructure only:
imported by the tests, the smoke check and the benchmark's CPU-baseline leg,
never by the library or its Python binding."""
