"""CPU oracle for the AMXFP4 hot path. Test infrastructure only: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg, never by the GPU library or its Python binding."""
