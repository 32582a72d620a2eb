"""Oracle for the synchronisation subsystem (test infrastructure only).

Pure-Python restatement of the paper's index formulas and wave arithmetic, plus a
small event-driven simulator of tiles running on a fixed number of execution
slots.  Shares nothing with the GPU library.

Conventions follow Fig. 4 of the paper: a tile is (x, y) in a grid (gx, gy); x
runs over column tiles of the output, y over row tiles.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Callable, Dict, List, Sequence, Tuple

Tile = Tuple[int, int]
Grid = Tuple[int, int]


# ---- tile order and policies (Fig. 4b) ------------------------------------

def row_major(tile: Tile, grid: Grid) -> int:
    """RowMajor order: all x of a row first, then the next y."""
    x, y = tile
    return y * grid[0] + x


def tilesync_sem(tile: Tile, grid: Grid) -> int:
    """TileSync: a distinct semaphore for each producer tile."""
    x, y = tile
    return x * grid[1] + y


def tilesync_value(tile: Tile, grid: Grid) -> int:
    return 1


def rowsync_sem(tile: Tile, grid: Grid) -> int:
    """RowSync: all tiles of one row share a semaphore."""
    return tile[1]


def rowsync_value(tile: Tile, grid: Grid) -> int:
    """A row is ready when each of its grid.x column tiles has posted."""
    return grid[0]


def stridedsync_sem(tile: Tile, grid: Grid, stride: int) -> int:
    """StridedSync (Section IV-B, attention): the tiles x, x+stride, x+2*stride, ... of a
    row share one semaphore; there are `stride` semaphores per row."""
    x, y = tile
    return y * stride + (x % stride)


def stridedsync_value(tile: Tile, grid: Grid, stride: int) -> int:
    """Number of tiles mapped onto one semaphore (3 for Q, K, V)."""
    return grid[0] // stride


# ---- wave model (Section II-A, Table I) ------------------------------------

def tbs_per_wave(occupancy: int, n_sm: int) -> int:
    return occupancy * n_sm


def waves(n_tbs: int, occupancy: int, n_sm: int) -> float:
    """Fractional wave count as Table I prints it (e.g. 192 / 160 = 1.2)."""
    return n_tbs / tbs_per_wave(occupancy, n_sm)


def wave_count(n_tbs: int, occupancy: int, n_sm: int) -> int:
    """ceil(TBs / (occupancy * SMs))."""
    return math.ceil(n_tbs / tbs_per_wave(occupancy, n_sm))


def utilization(n_tbs: int, occupancy: int, n_sm: int) -> float:
    """Table I's utilisation column: thread blocks over the slots of all waves run."""
    return n_tbs / (wave_count(n_tbs, occupancy, n_sm) * tbs_per_wave(occupancy, n_sm))


# ---- number of synchronisations (Section III-E) ----------------------------

def sync_count(policy: str, prod_grid: Grid, cons_grid: Grid) -> int:
    """Semaphore waits of a GeMM->GeMM chain where each consumer tile reads a full row of
    producer tiles and consumer row tiles coincide with producer row tiles."""
    n_cons = cons_grid[0] * cons_grid[1]
    if policy == "tile":
        return n_cons * prod_grid[0]
    if policy == "row":
        return n_cons
    raise ValueError(policy)


# ---- schedule simulator ----------------------------------------------------

@dataclass
class SimTile:
    stage: int                 # 0 = producer, 1 = consumer, ...
    duration: float
    deps: Sequence[int]        # indices (into the issue-ordered list) this tile waits on


def simulate(n_slots: int, tiles: List[SimTile], stream_sync: bool) -> float:
    """Makespan of `tiles` issued in list order onto `n_slots` execution slots.

    A tile is issued to the earliest free slot.  With stream_sync a tile of stage s may not
    be issued before every tile of stage s-1 has finished.  Without it the tile occupies its
    slot from issue, starts computing once all its deps have finished, and frees the slot
    when done (it spins while holding the slot, as a waiting thread block does).
    """
    free_at = [0.0] * n_slots
    finish: List[float] = [0.0] * len(tiles)
    stage_end: Dict[int, float] = {}
    for i, t in enumerate(tiles):
        slot = min(range(n_slots), key=lambda s: free_at[s])
        issue = free_at[slot]
        if stream_sync and t.stage > 0:
            issue = max(issue, stage_end.get(t.stage - 1, 0.0))
        start = issue
        for dep in t.deps:
            assert dep < i, "dependencies must be issued earlier"
            start = max(start, finish[dep])
        finish[i] = start + t.duration
        free_at[slot] = finish[i]
        stage_end[t.stage] = max(stage_end.get(t.stage, 0.0), finish[i])
    return max(finish) if finish else 0.0


def gemm_chain_tiles(prod_grid: Grid, cons_grid: Grid, prod_dur: float = 1.0,
                     cons_dur: float = 1.0,
                     rows_per_cons_row: Callable[[int], Sequence[int]] = None) -> List[SimTile]:
    """Producer tiles then consumer tiles, both in row-major order; consumer tile (x, y)
    depends on every producer tile of the producer rows it reads (default: row y)."""
    tiles: List[SimTile] = []
    pidx: Dict[Tile, int] = {}
    for y in range(prod_grid[1]):
        for x in range(prod_grid[0]):
            pidx[(x, y)] = len(tiles)
            tiles.append(SimTile(0, prod_dur, ()))
    for y in range(cons_grid[1]):
        prow = rows_per_cons_row(y) if rows_per_cons_row else (y,)
        deps = [pidx[(x, yy)] for yy in prow for x in range(prod_grid[0])]
        for _x in range(cons_grid[0]):
            tiles.append(SimTile(1, cons_dur, deps))
    return tiles
