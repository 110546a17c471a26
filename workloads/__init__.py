"""Seeded synthetic workload generators (no arithmetic of the method)."""
