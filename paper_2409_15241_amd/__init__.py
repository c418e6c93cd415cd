"""MI355X-native rank-local hot path of Domino tensor-parallel training.

``paper_2409_15241_amd.domino`` is the ctypes binding of the C-ABI library built
from ``csrc/``; ``paper_2409_15241_amd.synth`` draws the seeded synthetic inputs.
Nothing is loaded at package import time.
"""
__all__ = ["domino", "synth"]
