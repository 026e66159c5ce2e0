"""Seeded synthetic inputs and workload shape tables (no arithmetic of the method)."""
