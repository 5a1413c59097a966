"""CPU oracle of the MixLLM quantized linear layer.  Test infrastructure only:
imported by tests/, the smoke check and the benchmark's cpu_baseline leg."""
