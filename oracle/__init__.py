"""fp64 CPU oracle of the gated Multi-Head FFN.  Test infrastructure only:
imported by tests, the smoke check and the bench's cpu_baseline leg, never by
the GPU library or its Python binding."""
