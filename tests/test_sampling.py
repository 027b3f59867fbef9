"""The token sampling of the full-size GPU parity tests (host logic only)."""
import numpy as np

from gpu_util import tile_covering_tokens


def test_tile_covering_tokens_cover_every_tile():
    offsets = np.array([0, 3, 3, 43, 43 + 130])
    perm = np.arange(173) * 2            # pair ids: token = pair // k with k = 2
    toks = tile_covering_tokens(offsets, perm, 2)
    pos = [t for t in toks]              # token == sorted position here
    assert sum(0 <= q < 3 for q in pos) == 1
    assert sorted((q - 3) // 16 for q in pos if 3 <= q < 43) == [0, 1, 2]
    assert sorted((q - 43) // 16 for q in pos if q >= 43) == list(range(9))
