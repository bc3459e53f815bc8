"""MI355X-native decoder-layer hot path (forward, backward, gradient-shard accumulation, weight
staging) for weight-pipeline training.  The compute lives in the HIP library under csrc/;
`binding` is the thin ctypes layer over its C ABI and `inputs` the seeded synthetic data."""
