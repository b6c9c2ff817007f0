"""Column locality of predicted masks: how many fetches of the second operand (key rows for Q K^T,
value rows for A V) a row-parallel dataflow saves over row-by-row processing (paper section 5.2,
figure 11, table 4).  Test / analysis infrastructure on the CPU: it reads masks made by the oracle.

Model (the paper's figure 11): P processing elements work on P consecutive attention rows, one kept
position per element and step.  An operand row fetched in a step serves every element that
processes that key in the same step.
  row-by-row                  every kept position fetches its operand row: P * keep fetches per tile
  row-parallel, in order      every element walks its list in ascending key order; a step fetches the
                              distinct keys met in it
  row-parallel, reordered     elements may take their keys in any order.  `greedy`: in every step the
                              key wanted by most idle elements is fetched for all of them, until
                              every element is busy (a feasible schedule); `union`: distinct keys of
                              the tile, the floor no schedule can beat.
The reduction factor is row-by-row fetches divided by the dataflow's fetches (table 4 reports it)."""
from __future__ import annotations

import numpy as np


def fetches_in_order(tile: np.ndarray) -> int:
    """tile: [P, keep] ascending key lists.  Distinct keys per step, summed over steps."""
    return int(sum(len(np.unique(tile[:, t])) for t in range(tile.shape[1])))


def fetches_union(tile: np.ndarray) -> int:
    return int(len(np.unique(tile)))


def fetches_greedy(tile: np.ndarray) -> int:
    """A feasible reordered schedule: per step, keys by falling demand among the still idle elements."""
    want = [set(row.tolist()) for row in tile]
    fetches = 0
    while any(want):
        idle = {p for p, w in enumerate(want) if w}
        demand: dict[int, list[int]] = {}
        for p in idle:
            for j in want[p]:
                demand.setdefault(j, []).append(p)
        # keys by demand at the start of the step; an element takes the first of them it still wants
        for j, ps in sorted(demand.items(), key=lambda kv: (-len(kv[1]), kv[0])):
            takers = [p for p in ps if p in idle]
            if not takers:
                continue
            fetches += 1
            for p in takers:
                idle.discard(p)
                want[p].discard(j)
            if not idle:
                break
    return fetches


def reduction_factors(idx: np.ndarray, rows_per_unit: int, P: int, max_tiles: int = 64, seed: int = 0) -> dict:
    """idx: [units, keep] mask of one head (ascending lists); rows_per_unit: 1 or 8 (rows of a unit share
    a list).  Samples up to max_tiles tiles of P consecutive attention rows."""
    units, keep = idx.shape
    rows = units * rows_per_unit
    tiles = rows // P
    rng = np.random.default_rng(seed)
    pick = np.arange(tiles) if tiles <= max_tiles else np.sort(rng.choice(tiles, max_tiles, replace=False))
    base = in_order = greedy = union = 0
    for t in pick:
        r = np.arange(t * P, (t + 1) * P)
        tile = idx[r // rows_per_unit]
        base += P * keep
        in_order += fetches_in_order(tile)
        greedy += fetches_greedy(tile)
        union += fetches_union(tile)
    return dict(P=P, tiles=len(pick), in_order=base / in_order, reordered_greedy=base / greedy,
                reordered_floor=base / union)


def main():
    import sys
    from pathlib import Path
    sys.path.insert(0, str(Path(__file__).resolve().parent.parent))
    import dsa_inputs as di
    from oracle import dsa_oracle
    print("| workload | rows per tile | in order | reordered (greedy schedule) | reordered (floor: distinct keys) |")
    print("|---|---|---|---|---|")
    for name in ("C4f", "C4v", "C5"):
        cfg = di.CONFIGS[name]
        x = di.make_inputs(cfg)
        Qt = x.Qt.reshape(cfg.N, cfg.L, cfg.k)[:1]
        Kt = x.Kt.reshape(cfg.N, cfg.L, cfg.k)[:1]
        idx = dsa_oracle.predict_mask(Qt, Kt, cfg.keep, cfg.vec).reshape(-1, cfg.keep)
        for P in (4, 8, 16, 64):
            f = reduction_factors(idx, cfg.vec, P, max_tiles=24)
            print(f"| {name} | {P} | {f['in_order']:.2f}x | {f['reordered_greedy']:.2f}x | {f['reordered_floor']:.2f}x |", flush=True)


if __name__ == "__main__":
    main()
