"""TEST INFRASTRUCTURE: float64 CPU oracle (graph forward/BPTT and brute-force schedule).
Only tests, the smoke entry and the benchmark's CPU-baseline leg may import this package."""
