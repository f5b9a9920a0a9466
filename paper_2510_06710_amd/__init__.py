"""MI355X-native batched VLA rollout step and log-prob recompute (HIP kernels behind a C ABI).

``binding`` mirrors include/vla.h one to one; ``harness`` owns device buffers for tests and the
benchmark.  Nothing here computes on the CPU: without the built library every call raises."""
