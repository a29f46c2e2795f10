"""Seeded synthetic input generators (no attention / cache arithmetic lives here)."""
