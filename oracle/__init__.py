"""Test infrastructure: the CPU oracle.  Not part of the product path."""
