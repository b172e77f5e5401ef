"""Seeded synthetic input generators shared by the oracle's tests and the GPU tests."""
from .configs import BASE_SEED, CONFIGS, dense_to_csr, make  # noqa: F401
