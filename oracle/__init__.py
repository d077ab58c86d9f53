"""CPU reference implementation used only by tests, the smoke check and the benchmark's
CPU-baseline leg.  Nothing in the GPU library imports this package."""
