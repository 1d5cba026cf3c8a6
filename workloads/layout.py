"""Arrange one generated batch as the flat arrays a merged hash table consumes.

Pure data movement: concatenation of the per-feature ID lists that map to one merged table,
their offsets, and the logical-table index of each field.  The plan (which logical table goes to
which merged table) is an argument; it is computed by the library under test or by the checker.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np


def merged_inputs(features, ids: Sequence[np.ndarray], merged_of: Sequence[int], g: int
                  ) -> Tuple[np.ndarray, np.ndarray, np.ndarray, List[int]]:
    """Flat raw IDs (field-major), field offsets [F+1], field tags [F] and the feature indices
    of merged table ``g``."""
    sel = [i for i, f in enumerate(features) if merged_of[f.table] == g]
    parts = [np.ascontiguousarray(ids[i], dtype=np.uint64) for i in sel]
    x = np.concatenate(parts) if parts else np.zeros(0, dtype=np.uint64)
    off = np.zeros(len(sel) + 1, dtype=np.int64)
    off[1:] = np.cumsum([len(p) for p in parts])
    tags = np.array([features[i].table for i in sel], dtype=np.uint8)
    return x, off, tags, sel
