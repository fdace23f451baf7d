"""Counter-based random streams keyed by (seed, tensor name).

Every tensor of a synthetic SuperNet is drawn from its own Philox stream whose
key is a stable hash of the seed and the tensor's name, so any consumer can
regenerate exactly the same bits for one tensor without generating the others.
"""
import hashlib

import numpy as np


def keyed_rng(seed: int, name: str) -> np.random.Generator:
    digest = hashlib.sha256(f"{int(seed)}:{name}".encode()).digest()
    key = int.from_bytes(digest[:16], "little")
    return np.random.Generator(np.random.Philox(key=key))
