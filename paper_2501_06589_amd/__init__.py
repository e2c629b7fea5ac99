"""MI355X-native Ladder-Residual shard forward (hand-written HIP behind a C-ABI).

``inputs`` (seeded synthetic inputs) imports nothing from the HIP path; the
binding in ``ladder`` loads the compiled library on first use and raises if it
is missing.
"""
__all__ = ["inputs", "ladder"]
