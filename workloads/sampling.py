"""Which permuted query rows a sampled check looks at (harness logic only: no arithmetic of the
method). At full size a CPU check can afford only some rows of a head; random rows alone reach
the rows where an implementation is most likely to go wrong -- the edges of clusters and of
fixed-height row tiles, the smallest and largest cluster, rows with nothing or with the most
routed -- only by luck, so those are always taken, each under a name a failing check can print.
"""
from __future__ import annotations

from typing import Dict, Sequence

import numpy as np


def structural_rows(q_offsets: np.ndarray, row_ptr: np.ndarray, Cq: int, rng: np.random.Generator,
                    n_random: int = 48, tile_heights: Sequence[int] = (384, 256, 128)) -> Dict[str, int]:
    """Named permuted row positions of one head.

    q_offsets [Cq+2]: cluster a is rows [q_offsets[a], q_offsets[a+1]); the tail (text rows) is
    [q_offsets[Cq], q_offsets[Cq+1]). row_ptr [>= Cq+1]: routed key clusters per query cluster
    (CSR). tile_heights: row-tile heights an implementation may cut a cluster into; for each, the
    last row of a full tile and the first row of the next one are taken inside the largest cluster.
    """
    q_offsets = np.asarray(q_offsets, np.int64)
    sizes = np.diff(q_offsets[: Cq + 1])
    n_rows = int(q_offsets[Cq + 1])
    live = np.flatnonzero(sizes > 0)
    out: Dict[str, int] = {}
    if live.size:
        small = int(live[np.argmin(sizes[live])])
        large = int(live[np.argmax(sizes[live])])
        for tag, a in (("smallest cluster", small), ("largest cluster", large)):
            out[f"first row of the {tag} ({a}, {int(sizes[a])} rows)"] = int(q_offsets[a])
            out[f"last row of the {tag} ({a}, {int(sizes[a])} rows)"] = int(q_offsets[a + 1] - 1)
        for th in tile_heights:
            if sizes[large] > th:
                out[f"last row of the first {th}-row tile of cluster {large}"] = int(q_offsets[large] + th - 1)
                out[f"first row of the second {th}-row tile of cluster {large}"] = int(q_offsets[large] + th)
            full = (int(sizes[large]) // th) * th
            if 0 < full < sizes[large]:
                out[f"first row of the partly filled last {th}-row tile of cluster {large}"] = int(q_offsets[large] + full)
        # last partly filled group of 32 / 64 rows of the largest cluster
        for w in (32, 64):
            full = (int(sizes[large]) // w) * w
            if 0 < full < sizes[large]:
                out[f"first row of the last partial group of {w} of cluster {large}"] = int(q_offsets[large] + full)
        n_routed = np.diff(np.asarray(row_ptr, np.int64)[: Cq + 1])
        none = [int(a) for a in live if n_routed[a] == 0]
        if none:
            out[f"a row of cluster {none[0]} with nothing routed"] = int(q_offsets[none[0]] + sizes[none[0]] // 2)
        most = int(live[np.argmax(n_routed[live])])
        out[f"a row of cluster {most} with the most routed key clusters ({int(n_routed[most])})"] = \
            int(q_offsets[most] + sizes[most] // 2)
        fewest = int(live[np.argmin(n_routed[live])])
        out[f"a row of cluster {fewest} with the fewest routed key clusters ({int(n_routed[fewest])})"] = \
            int(q_offsets[fewest] + sizes[fewest] // 2)
    n_tail = int(q_offsets[Cq + 1] - q_offsets[Cq])
    if n_tail:
        out["first tail (text) row"] = int(q_offsets[Cq])
        out["last tail (text) row"] = n_rows - 1
    out["row 0"] = 0
    out["last row"] = n_rows - 1
    for i, p in enumerate(rng.choice(n_rows, size=min(n_random, n_rows), replace=False)):
        out[f"random row #{i}"] = int(p)
    return out
