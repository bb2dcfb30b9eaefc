"""Seeded synthetic input generators (no method arithmetic); see gen.py."""
