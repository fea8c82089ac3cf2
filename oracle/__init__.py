"""Test infrastructure: the CPU fp64 oracle. Never imported by the product path."""
