"""Seeded synthetic inputs shared by the oracle-side and GPU-side tests and by the bench."""
