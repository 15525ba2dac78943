"""Seeded synthetic cost tables (integer nanoseconds per match).

They stand in for the measurer M of paper Sec. 4.2 in CPU-only tests of the
placement search: a table is just one int64 per enumerated match.  `ties`
draws costs from a handful of values so that many placements share the optimal
total and the canonical tie-break is exercised.
"""
from __future__ import annotations

import numpy as np


def synthetic_costs(n_matches: int, seed: int, match_sizes=None,
                    ties: bool = False) -> np.ndarray:
    rng = np.random.default_rng([int(seed), 424243])
    if ties:
        c = rng.integers(1, 4, n_matches).astype(np.int64) * 1000
    else:
        c = rng.integers(500, 20000, n_matches).astype(np.int64)
    if match_sizes is not None and not ties:
        # a fused match usually costs less than the sum of its parts but more
        # than one part: scale with a sub-linear function of the group size
        s = np.asarray(match_sizes, dtype=np.float64)
        c = (c * (1.0 + 0.35 * (s - 1.0))).astype(np.int64)
    return c
