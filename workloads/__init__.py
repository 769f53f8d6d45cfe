"""Seeded synthetic inputs shared by the oracle's tests and the HIP path's tests."""
