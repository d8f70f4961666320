"""Seeded synthetic input generators (shared by the oracle tests and the GPU path)."""
from .generators import *  # noqa: F401,F403
from .generators import make_config, CONFIG_NAMES  # noqa: F401
