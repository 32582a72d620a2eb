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


# ---- forward progress under a dispatch order (Section III-B) ----------------

def simulate_dispatch(n_slots: int, tiles: List[SimTile], dispatch: Sequence[int], by_ticket: bool,
                      spin_limit: float = None):
    """Workgroups started in the order `dispatch` (a permutation of range(len(tiles))) on `n_slots` slots.

    by_ticket=False: workgroup i runs tile i (tiles named by the block index).  A workgroup holds
    its slot from its start; it computes once every dependency has finished, and spins until then.
    If the tiles it waits for belong to workgroups that cannot start because spinning workgroups
    hold every slot, nothing moves any more: Section III-B's deadlock.
    by_ticket=True: whatever workgroup starts next takes the next tile of the list (all tiles of a
    stage before the next stage's), so a spinning workgroup's dependencies are always held by
    workgroups that have already started.
    spin_limit: a wait longer than this is given up (the tile then finishes at once, marked
    timed out, as the library's bounded wait does); None = wait for ever.

    Returns (makespan or None if deadlocked, number of tiles that timed out).
    """
    n = len(tiles)
    assert sorted(dispatch) == list(range(n))
    finish = [None] * n            # finish time of tile i once known
    started = {}                   # tile -> (slot start time)
    waiting = []                   # started tiles whose finish time is not known yet
    free_at = [0.0] * n_slots      # when each slot is free again (inf while held by an unresolved workgroup)
    INF = float("inf")
    next_wg, ticket, timed_out = 0, 0, 0

    def resolve():
        """Fix the finish time of every started tile whose dependencies' finish times are known."""
        nonlocal timed_out
        progress = True
        while progress:
            progress = False
            for t in list(waiting):
                deps = tiles[t].deps
                if all(finish[d] is not None for d in deps):
                    ready = max([started[t][0]] + [finish[d] for d in deps])
                    if spin_limit is not None and ready - started[t][0] > spin_limit:
                        ready = started[t][0] + spin_limit
                        finish[t] = ready           # gives up: no work done, its post still goes out
                        timed_out += 1
                    else:
                        finish[t] = ready + tiles[t].duration
                    free_at[started[t][1]] = finish[t]
                    waiting.remove(t)
                    progress = True

    while next_wg < n:
        slot = min(range(n_slots), key=lambda s: free_at[s])
        if free_at[slot] == INF:
            # every slot is held by a workgroup whose dependencies have not even started
            if spin_limit is None:
                return None, timed_out
            # bounded waits: the longest-waiting workgroup gives up first
            t = min(waiting, key=lambda w: started[w][0])
            finish[t] = started[t][0] + spin_limit
            free_at[started[t][1]] = finish[t]
            waiting.remove(t)
            timed_out += 1
            resolve()
            continue
        tile = ticket if by_ticket else dispatch[next_wg]
        ticket += 1
        next_wg += 1
        started[tile] = (free_at[slot], slot)
        free_at[slot] = INF
        waiting.append(tile)
        resolve()
    resolve()
    if waiting:
        if spin_limit is None:
            return None, timed_out
        while waiting:
            t = min(waiting, key=lambda w: started[w][0])
            finish[t] = started[t][0] + spin_limit
            free_at[started[t][1]] = finish[t]
            waiting.remove(t)
            timed_out += 1
            resolve()
    return max(f for f in finish if f is not None), timed_out
