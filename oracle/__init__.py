"""fp64 CPU oracle of the ResNet-50 training-step path.  Test infrastructure only:
imported by tests/, the smoke check and the benchmark's cpu_baseline leg, never by the product."""
