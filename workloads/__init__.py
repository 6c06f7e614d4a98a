"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This package holds input recipes only: no step of the decomposition lives here.
"""
