"""CPU oracle of the quantized-linear path: test infrastructure, never used by the GPU library."""
