"""Test infrastructure: the double-precision CPU reference (see oracle.py)."""
