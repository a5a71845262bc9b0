"""Brute-force statement of the tiling cost model and of the tile assignment.  TEST INFRASTRUCTURE ONLY.

Section 4.2 ("Shape tiling"): a candidate tile size t over a space of ``total`` elements run on N
cores costs  ceil(#tiles / N) * (t + 2)  with  #tiles = ceil(total / t); hardware_align_div takes
the minimum-cost tile size not above T_max and rounds it up to the hardware access width, still
not above T_max; the tail tile is not padded.  Algorithm 2, the two statements that compute m and
the tile range of a core, give the tile-to-core assignment.

Readings where the paper is silent: all candidate sizes 1..T_max compete even when the whole space
already fits T_max (the worked example splits a tensor that fits); ties go to the larger tile
(fewer tiles); the "+2" is in elements.  Everything here is the definition evaluated exhaustively.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple


def ceil_div(a: int, b: int) -> int:
    return -(-a // b)


def tile_cost(total: int, t: int, n_cores: int, extra: int = 2) -> int:
    """Bottleneck workload of all cores for tile size t (Section 4.2, the cost formula)."""
    tiles = ceil_div(total, t)
    return ceil_div(tiles, n_cores) * (t + extra)


def min_cost_tile(total: int, n_cores: int, t_max: int, extra: int = 2) -> int:
    """The minimum-cost tile size in 1..min(T_max, total), by exhaustive search; ties -> larger."""
    best_t, best_c = None, None
    for t in range(1, min(t_max, total) + 1):
        c = tile_cost(total, t, n_cores, extra)
        if best_c is None or c <= best_c:
            best_t, best_c = t, c
    return best_t


def align_up_capped(t: int, align: int, t_max: int) -> int:
    """Round t up to a multiple of ``align`` without exceeding T_max (fall back to the largest
    multiple below T_max, or to t itself if not even one aligned size fits)."""
    up = ceil_div(t, align) * align
    if up <= t_max:
        return up
    down = (t_max // align) * align
    return down if down >= align else t


def hardware_align_div(total: int, n_cores: int, t_max: int, align: int, extra: int = 2) -> Tuple[int, int]:
    """Returns (minimum-cost tile size, that size rounded up to the hardware width)."""
    t = min_cost_tile(total, n_cores, t_max, extra)
    return t, align_up_capped(t, align, t_max)


def tiles_of(total: int, t: int) -> List[Tuple[int, int]]:
    """[start, end) of every tile; the last one is the unpadded tail."""
    return [(s, min(total, s + t)) for s in range(0, total, t)]


def vm_tile_range(n_tiles: int, n_cores: int, core_id: int) -> Tuple[int, int]:
    """Algorithm 2: m = ceil(M/N); core ``id`` runs tiles [m*id, min(M, m*(id+1)))."""
    m = ceil_div(n_tiles, n_cores)
    lo = m * core_id
    hi = min(n_tiles, m * (core_id + 1))
    return lo, max(lo, hi)


def interleaved_tiles(n_tiles: int, n_cores: int, core_id: int) -> List[int]:
    """The round-robin alternative to Algorithm 2's blocked range that the library uses by default on the
    GPU: core ``id`` runs tiles id, id + N, id + 2N, ...  Like the blocked range it is static, needs no
    atomics and gives every core ceil(M/N) tiles or one fewer."""
    return list(range(core_id, n_tiles, n_cores))


def shape_tiling(dominant_shape: Sequence[int], t_max: int, n_cores: int, align: int,
                 extra: int = 2) -> List[int]:
    """Algorithm 1 for one dominant shape: walk the dimensions from the outermost inwards; a
    dimension whose inner remainder still exceeds T_max gets tile extent 1; the first dimension
    whose inner remainder fits is split by the cost model; all inner dimensions stay whole.
    Returns the tile extent per dimension.  (Other ops' shapes take the same extent on that
    dimension unless theirs is 1 there: broadcast or reduced dimensions are skipped.)"""
    dims = list(dominant_shape)
    tile = list(dims)
    size = 1
    for d in dims:
        size *= d
    outer_tiles = 1
    for i, ell in enumerate(dims):
        inner = size // ell
        if inner > t_max:
            tile[i] = 1
            outer_tiles *= ell
            size = inner
            continue
        # candidates: t slices of this dimension per tile, tile size t*inner <= T_max
        best_t, best_c = None, None
        for t in range(1, min(ell, max(1, t_max // inner)) + 1):
            n_tiles = outer_tiles * ceil_div(ell, t)
            c = ceil_div(n_tiles, n_cores) * (t * inner + extra)
            if best_c is None or c <= best_c:
                best_t, best_c = t, c
        t = best_t
        if inner == 1:
            t = align_up_capped(t, align, t_max)
        tile[i] = min(t, ell)      # a tile never exceeds the dimension: the tail is not padded
        break
    return tile
