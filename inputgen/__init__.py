"""Seeded synthetic input generator (serves the HIP path and the oracle; holds no method arithmetic)."""
