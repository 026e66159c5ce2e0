"""CPU oracle (test infrastructure only).  Never imported by the HIP path or its binding;
only tests, the smoke check and the benchmark's cpu_baseline leg use it."""
