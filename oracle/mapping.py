"""Oracle for the tile-centric mappings and tile schedules (test infrastructure only).

Static mapping: the affine formulas the paper gives for AllGather(pull)+GEMM in
its "Tile-Centric Mapping" section (shape map f_S, rank map f_R, channel map
f_C), evaluated literally, one producer tile at a time.  The consumer map is
only said to be "similar"; the reading taken here: a consumer tile waits on
every channel whose row range it touches.

Everything in this file is integer work and is compared bit-exactly with what
the library reports through its schedule dump.
"""
from __future__ import annotations

import math

XCDS = 8  # accelerator complex dies of the target GPU; workgroup w runs on die w % 8


def ceil_div(a: int, b: int) -> int:
    return -(-a // b)


# ---------------------------------------------------------------------------
# Static mapping, "Tile-Centric Mapping" section, the displayed equation
# ---------------------------------------------------------------------------

def producer_tile(tile_id_p: int, M: int, R: int, C: int, Tm_p: int):
    """Shape range, source rank and channel of one producer (AllGather) row tile."""
    M_per_rank = math.ceil(M / R)
    M_per_channel = math.ceil(M / (R * C))
    range_M = (tile_id_p * Tm_p, tile_id_p * Tm_p + Tm_p)
    src_rank = tile_id_p // (M_per_rank // Tm_p)
    channel = tile_id_p // (M_per_channel // Tm_p)
    return range_M, src_rank, channel


def producer_table(M: int, R: int, C: int, Tm_p: int):
    """All producer row tiles: list of (row_lo, row_hi, src_rank, channel)."""
    out = []
    for t in range(ceil_div(M, Tm_p)):
        (lo, hi), s, c = producer_tile(t, M, R, C, Tm_p)
        out.append((lo, hi, s, c))
    return out


def channel_expected(M: int, K: int, R: int, C: int, Tm_p: int, Tn_p: int) -> int:
    """Producer tiles that must finish before a channel is ready: the row tiles
    inside the channel times the column tiles a row tile is cut into."""
    M_per_channel = math.ceil(M / (R * C))
    return (M_per_channel // Tm_p) * ceil_div(K, Tn_p)


def consumer_tile(tile_id_c: int, M: int, N: int, R: int, C: int, Tm_c: int, Tn_c: int):
    """(bm, bn, row_lo, row_hi, chan_lo, chan_hi) of a GEMM output tile; channels
    are the global indices of the equation (rank * C + local channel); the tile
    waits on chan_lo..chan_hi inclusive."""
    nbn = ceil_div(N, Tn_c)
    bm, bn = divmod(tile_id_c, nbn)
    lo = bm * Tm_c
    hi = min(lo + Tm_c, M)
    M_per_channel = math.ceil(M / (R * C))
    return bm, bn, lo, hi, lo // M_per_channel, (hi - 1) // M_per_channel


# ---------------------------------------------------------------------------
# Tile order: which output tile a persistent workgroup computes at schedule
# position p.  Workgroup w of a grid of G takes positions w, w+G, w+2G, ...
# ---------------------------------------------------------------------------

def arrival_rows(nbm: int, R: int, first_rank: int):
    """Row blocks in the order in which they are complete when every other
    rank sends its shard over a link of its own, all links side by side: the
    blocks of `first_rank` (the local shard, nothing to send), then block j of
    first_rank+1, first_rank+2, ... before block j+1 of any."""
    bpr = nbm // R
    rows = [first_rank * bpr + j for j in range(bpr)]
    for j in range(bpr):
        for q in range(1, R):
            rows.append(((first_rank + q) % R) * bpr + j)
    return rows


def logical_order(nbm: int, nbn: int, R: int, first_rank: int, rotate: bool, group_m: int = 1, arrival: bool = False):
    """Row-blocks in natural order, or rotated so that the row-blocks owned by
    `first_rank` come first and the other ranks follow in ring order, or (with
    `arrival`, if R divides nbm and R > 1) in arrival order.  The row blocks
    are then taken in groups of `group_m`; inside a group all row blocks of
    one column block come before the next column block."""
    blocks_per_rank = nbm // R if rotate else 0
    rows = [(i + first_rank * blocks_per_rank) % nbm if rotate else i for i in range(nbm)]
    if arrival and rotate and nbm % R == 0 and R > 1:
        rows = arrival_rows(nbm, R, first_rank)
    order = []
    for start in range(0, nbm, group_m):
        group = rows[start:start + group_m]
        for bn in range(nbn):
            for bm in group:
                order.append(bm * nbn + bn)
    return order


def xcd_positions(n_tiles: int, G: int, busy_first: bool = False):
    """position -> logical index.  Inside each full round of G positions the
    workgroups that share a die (w % 8) are given a contiguous run of G/8
    logical tiles, so tiles that run side by side on one die share operands.
    A ragged last round gets the same treatment if its length is a multiple of
    8, else it is left in order.  With G not a multiple of 8 nothing moves.

    `busy_first` (tile order is a free choice of the design space; this one is
    for consumers whose first tiles wait for data that arrives in logical
    order): if the last round is a partial one of `tail` positions (a multiple
    of 8, more than one round in all), the workgroups w < tail are the ones
    with a tile more than the others, so in round 0 they take the logical
    tiles [0, tail) -- the earliest data -- and the workgroups with a tile
    less take [tail, G); both sets again as one contiguous run per die."""
    pos = []
    tail = n_tiles % G
    for p in range(n_tiles):
        rnd, w = divmod(p, G)
        span = min(G, n_tiles - rnd * G)
        if busy_first and G % XCDS == 0 and rnd == 0 and n_tiles > G and tail and tail % XCDS == 0:
            die, i, tb = w % XCDS, w // XCDS, tail // XCDS
            pos.append(die * tb + i if i < tb else tail + die * ((G - tail) // XCDS) + (i - tb))
        elif G % XCDS == 0 and span % XCDS == 0:
            per_die = span // XCDS
            pos.append(rnd * G + (w % XCDS) * per_die + w // XCDS)
        else:
            pos.append(p)
    return pos


def tile_schedule(nbm: int, nbn: int, R: int, first_rank: int, rotate: bool, G: int, swizzle: bool, group_m: int = 1, arrival: bool = False,
                  busy_first: bool = False):
    """Output-tile id at every schedule position."""
    logical = logical_order(nbm, nbn, R, first_rank, rotate, group_m, arrival)
    n = nbm * nbn
    pos = xcd_positions(n, G, busy_first) if swizzle else list(range(n))
    return [logical[pos[p]] for p in range(n)]


def ag_gemm_schedule_records(M, N, K, R, C, rank, Tm_c, Tn_c, G, rotate=True, swizzle=True, group_m=1, arrival=False):
    """One 8-int record per schedule position:
    (tile_id, bm, bn, row_lo, row_hi, chan_lo, chan_hi, 0).  The consumer of an
    AllGather waits for rows that arrive in logical order, so its die swizzle
    is the `busy_first` one."""
    nbm, nbn = ceil_div(M, Tm_c), ceil_div(N, Tn_c)
    recs = []
    for t in tile_schedule(nbm, nbn, R, rank, rotate, G, swizzle, group_m, arrival, busy_first=True):
        bm, bn, lo, hi, clo, chi = consumer_tile(t, M, N, R, C, Tm_c, Tn_c)
        recs.append((t, bm, bn, lo, hi, clo, chi, 0))
    return recs


# ---------------------------------------------------------------------------
# GEMM + ReduceScatter: GEMM tiles are producers, reduce/push tiles consumers
# ---------------------------------------------------------------------------

def rs_tile_table(M, N, R, rank, Tm_c, Tn_c, Tm_r, Tn_r):
    """Reduce/push tiles of the partial product, row-major over (cm, cn):
    (cm, cn, row_lo, row_hi, col_lo, col_hi, dest_rank, expected) where
    expected = GEMM tiles that overlap the reduce tile and dest_rank = owner of
    its rows in the scattered output."""
    seg = M // R
    out = []
    for cm in range(ceil_div(M, Tm_r)):
        rlo, rhi = cm * Tm_r, min(cm * Tm_r + Tm_r, M)
        for cn in range(ceil_div(N, Tn_r)):
            clo, chi = cn * Tn_r, min(cn * Tn_r + Tn_r, N)
            n_m = (rhi - 1) // Tm_c - rlo // Tm_c + 1
            n_n = (chi - 1) // Tn_c - clo // Tn_c + 1
            out.append((cm, cn, rlo, rhi, clo, chi, rlo // seg, n_m * n_n))
    return out


def gemm_rs_schedule_records(M, N, K, R, rank, Tm_c, Tn_c, Tm_r, Tn_r, G, rotate=True, swizzle=True, group_m=1, own_first=False):
    """GEMM tiles in schedule order; with `rotate` the row-blocks of rank+1 come
    first and this rank's own segment last (ring order), so that pushes leave
    early and the segment that needs every peer's data is computed last; with
    `own_first` the own segment comes first and the ring follows.
    Record: (tile_id, bm, bn, row_lo, row_hi, cm_lo, cm_hi, cn_lo, cn_hi) where
    cm/cn ranges (inclusive) are the reduce tiles the GEMM tile notifies."""
    nbm, nbn = ceil_div(M, Tm_c), ceil_div(N, Tn_c)
    recs = []
    for t in tile_schedule(nbm, nbn, R, rank if own_first else (rank + 1) % R, rotate, G, swizzle, group_m):
        bm, bn = divmod(t, nbn)
        rlo, rhi = bm * Tm_c, min(bm * Tm_c + Tm_c, M)
        clo, chi = bn * Tn_c, min(bn * Tn_c + Tn_c, N)
        recs.append((t, bm, bn, rlo, rhi, rlo // Tm_r, (rhi - 1) // Tm_r, clo // Tn_r, (chi - 1) // Tn_r))
    return recs


def rs_consumer_order(M, N, R, rank, Tm_r, Tn_r, rotate=True, own_first=False):
    """Order in which reduce/push workgroups visit reduce tiles: same ring
    rotation of row blocks as the GEMM tiles (no die swizzle)."""
    ncm, ncn = ceil_div(M, Tm_r), ceil_div(N, Tn_r)
    return logical_order(ncm, ncn, R, rank if own_first else (rank + 1) % R, rotate)
