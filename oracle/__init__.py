"""TEST INFRASTRUCTURE ONLY: float64 CPU oracle for the circuit forward pass, PC flows and EM,
plus a plain-Python oracle of the layer compiler.  Only tests/, the smoke check and the
benchmark's cpu_baseline leg may import this package; the GPU library never does."""
