"""MI355X-native decode engine with in-flight weight updates: thin ctypes binding over libpl.so.

Every step of the hot path runs in the HIP library; this package only marshals arguments.
Importing the package does not load the library; the first call does, and fails loudly if it has
not been built (`python -m paper_2509_19128_amd.build`).
"""
from .binding import *  # noqa: F401,F403
