"""Seeded synthetic input generators (no decode-time arithmetic)."""
