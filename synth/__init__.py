"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This package holds shapes, seeds, random draws and bf16 bit packing only: none of
the decoder, sampler or weight-swap arithmetic lives here.
"""
from .inputs import *  # noqa: F401,F403
