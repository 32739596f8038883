"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark."""
from .mixes import SEED, BlockParams, Layer, Mix, Service, make_mix, make_vit_block  # noqa: F401
