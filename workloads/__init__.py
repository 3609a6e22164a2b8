"""Seeded synthetic workload generators (no method arithmetic)."""
