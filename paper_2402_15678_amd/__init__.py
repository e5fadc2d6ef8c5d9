"""MI355X-native verification step of aggregated speculative execution (Minions, arXiv 2402.15678).

The product is the HIP library behind ``include/minions_verify.h``; ``binding`` marshals arguments
to it and ``harness`` holds device buffers (PyTorch tensors) for tests and benchmarks."""
