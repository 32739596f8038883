"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark."""
from .mixes import SEED, Layer, Mix, Service, make_mix  # noqa: F401
