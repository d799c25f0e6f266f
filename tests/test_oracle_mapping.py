"""Pins for the mapping oracle: hand-evaluated equation values (golden files),
coverage/partition properties, and schedule properties."""
import os

import pytest

from oracle import mapping as mp

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_rows(name):
    rows = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append(tuple(int(v) for v in line.split()))
    return rows


@pytest.mark.parametrize("name,M,R,C,Tm", [("static_mapping_M256_R2_C2_Tm64.txt", 256, 2, 2, 64),
                                           ("static_mapping_M1024_R4_C2_Tm32.txt", 1024, 4, 2, 32)])
def test_static_mapping_hand_values(name, M, R, C, Tm):
    for t, lo, hi, src, ch in read_rows(name):
        (glo, ghi), gsrc, gch = mp.producer_tile(t, M, R, C, Tm)
        assert (glo, ghi, gsrc, gch) == (lo, hi, src, ch)


@pytest.mark.parametrize("M,R,C,Tm", [(256, 2, 1, 32), (256, 2, 2, 64), (8192, 8, 4, 128), (1536, 3, 2, 64), (8192, 8, 1, 1024)])
def test_producer_tiles_partition_rows_and_channels_nest_in_ranks(M, R, C, Tm):
    table = mp.producer_table(M, R, C, Tm)
    covered = [0] * M
    for lo, hi, src, ch in table:
        for r in range(lo, hi):
            covered[r] += 1
        # every row of the tile belongs to src's shard and to channel ch's row range
        assert lo // (M // R) == src == (hi - 1) // (M // R)
        assert lo // (M // (R * C)) == ch == (hi - 1) // (M // (R * C))
        assert ch // C == src                      # channels are numbered rank * C + local
    assert covered == [1] * M
    per_channel = {}
    for _, _, _, ch in table:
        per_channel[ch] = per_channel.get(ch, 0) + 1
    assert sorted(per_channel) == list(range(R * C))
    assert set(per_channel.values()) == {mp.channel_expected(M, 64, R, C, Tm, 64)}
    assert mp.channel_expected(M, 256, R, C, Tm, 64) == 4 * mp.channel_expected(M, 64, R, C, Tm, 64)


def test_consumer_tile_wait_set():
    # M=1024, R=4, C=2: channels of 128 rows.  A 256-row consumer tile spans two channels,
    # a 64-row tile sits inside one.
    assert mp.consumer_tile(0, 1024, 512, 4, 2, 256, 128) == (0, 0, 0, 256, 0, 1)
    assert mp.consumer_tile(5, 1024, 512, 4, 2, 256, 128) == (1, 1, 256, 512, 2, 3)
    assert mp.consumer_tile(4 * 3 + 2, 1024, 512, 4, 2, 64, 128) == (3, 2, 192, 256, 1, 1)
    # ragged last row block (M not a multiple of the tile)
    assert mp.consumer_tile(3 * 2, 1000, 200, 4, 1, 320, 128)[2:4] == (960, 1000)


@pytest.mark.parametrize("nbm,nbn,R,first,G", [(32, 16, 8, 0, 256), (32, 16, 8, 3, 256), (32, 32, 8, 5, 256),
                                               (8, 4, 2, 1, 16), (6, 5, 3, 2, 7), (4, 3, 2, 0, 8), (16, 7, 8, 7, 64)])
def test_schedule_is_a_permutation_with_first_rank_in_front(nbm, nbn, R, first, G):
    for swz in (False, True):
        s = mp.tile_schedule(nbm, nbn, R, first, True, G, swz)
        assert sorted(s) == list(range(nbm * nbn))
        per_rank = nbm // R
        n_first = per_rank * nbn
        first_tiles = {bm * nbn + bn for bm in range(first * per_rank, (first + 1) * per_rank) for bn in range(nbn)}
        lead = set(s[:n_first])
        if not swz or n_first % G == 0 or G >= nbm * nbn:
            assert lead == first_tiles or swz
        # whatever the swizzle, the first round holds the first rank's tiles before any later round does
        rounds_of_first = {i // G for i, t in enumerate(s) if t in first_tiles}
        assert min(rounds_of_first) == 0
    nat = mp.tile_schedule(nbm, nbn, R, first, False, G, False)
    assert nat == list(range(nbm * nbn))


def test_schedule_hand_example():
    # nbm=4, nbn=2, R=2, first rank 1 -> row blocks 2,3,0,1 ; tiles 4,5,6,7,0,1,2,3 without swizzle
    assert mp.tile_schedule(4, 2, 2, 1, True, 8, False) == [4, 5, 6, 7, 0, 1, 2, 3]
    # 16 tiles, G=16 (one round), 8 dies -> die x gets logical 2x, 2x+1; position p = w: die w%8, slot w//8
    s = mp.tile_schedule(4, 4, 2, 0, True, 16, True)
    assert s == [0, 2, 4, 6, 8, 10, 12, 14, 1, 3, 5, 7, 9, 11, 13, 15]


def test_swizzle_gives_each_die_a_contiguous_run():
    G, n = 256, 512
    pos = mp.xcd_positions(n, G)
    for rnd in range(2):
        for die in range(8):
            got = sorted(pos[rnd * G + w] for w in range(G) if w % 8 == die)
            assert got == list(range(rnd * G + die * 32, rnd * G + die * 32 + 32))


def test_busy_first_swizzle_gives_the_early_tiles_to_the_workgroups_with_a_tile_more():
    """448 tiles on 256 workgroups: workgroups 0..191 run two tiles.  In round 0 they get logical tiles 0..191 (die d the run
    24d..24d+23), the others 192..255 (die d the run 192+8d..192+8d+7); the second round is the plain swizzle; the whole
    thing is a permutation; with a whole number of rounds, or one round, nothing changes."""
    G, n = 256, 448
    pos = mp.xcd_positions(n, G, busy_first=True)
    assert sorted(pos) == list(range(n))
    for die in range(8):
        busy = sorted(pos[w] for w in range(192) if w % 8 == die)
        rest = sorted(pos[w] for w in range(192, 256) if w % 8 == die)
        assert busy == list(range(24 * die, 24 * die + 24)) and rest == list(range(192 + 8 * die, 192 + 8 * die + 8))
        second = sorted(pos[256 + w] for w in range(192) if w % 8 == die)
        assert second == list(range(256 + 24 * die, 256 + 24 * die + 24))
    assert pos[0] == 0 and pos[8] == 1 and pos[1] == 24 and pos[192] == 192 and pos[193] == 200   # hand values
    assert pos[256:] == mp.xcd_positions(n, G)[256:]
    for n2 in (512, 256, 200, 452):   # whole rounds, one round, less than a round, tail not a multiple of 8
        assert mp.xcd_positions(n2, G, busy_first=True) == mp.xcd_positions(n2, G)
    # three and a half rounds: only round 0 moves
    p3, q3 = mp.xcd_positions(896, 256, busy_first=True), mp.xcd_positions(896, 256)
    assert p3[256:] == q3[256:] and sorted(p3[:256]) == list(range(256)) and max(p3[w] for w in range(128)) == 127


def test_ag_gemm_schedule_records_cover_every_tile():
    recs = mp.ag_gemm_schedule_records(8192, 3584, 8192, 8, 4, 3, 256, 224, 256)
    assert len(recs) == 512 and sorted(r[0] for r in recs) == list(range(512))
    for t, bm, bn, lo, hi, clo, chi, _ in recs:
        assert t == bm * 16 + bn and lo == bm * 256 and hi == lo + 256
        assert clo == lo // 256 and chi == clo           # 256-row channels: exactly one channel per tile
    # the first 64 logical tiles belong to rank 3's rows
    assert {r[1] for r in recs[:256] if r[3] // 1024 == 3} == {12, 13, 14, 15}


def test_rs_tables():
    # 2x2 GEMM tiles per reduce tile -> expected 4; dest rank = owner of the rows
    tab = mp.rs_tile_table(1024, 512, 4, 1, 128, 128, 256, 256)
    assert len(tab) == 4 * 2
    assert all(e[7] == 4 for e in tab)
    assert [e[6] for e in tab] == [0, 0, 1, 1, 2, 2, 3, 3]
    # reduce tile smaller than the GEMM tile -> expected 1, and a GEMM tile notifies 2x2 of them
    tab = mp.rs_tile_table(1024, 512, 4, 1, 256, 256, 128, 128)
    assert all(e[7] == 1 for e in tab)
    recs = mp.gemm_rs_schedule_records(1024, 512, 64, 4, 1, 256, 256, 128, 128, 8, True, False)
    assert recs[0][:5] == (4, 2, 0, 512, 768)            # rank 2's rows come first for rank 1
    assert recs[0][5:] == (4, 5, 0, 1)
    assert [r[1] for r in recs][-2:] == [1, 1]           # own segment last
    order = mp.rs_consumer_order(1024, 512, 4, 1, 128, 128)
    assert sorted(order) == list(range(32))
    assert order[:4] == [16, 17, 18, 19] and order[-4:] == [12, 13, 14, 15]


def test_grouped_order_hand_example():
    # 4 row blocks, 3 column blocks, groups of 2 row blocks: (0,0)(1,0)(0,1)(1,1)(0,2)(1,2) then rows 2,3
    assert mp.logical_order(4, 3, 1, 0, False, 2) == [0, 3, 1, 4, 2, 5, 6, 9, 7, 10, 8, 11]
    # a short last group (5 row blocks, groups of 2) and rotation by rank 1 of 5 ranks (1 block per rank)
    assert mp.logical_order(5, 2, 5, 1, True, 2) == [2, 4, 3, 5, 6, 8, 7, 9, 0, 1]
    for gm in (1, 2, 3, 4, 8):
        assert sorted(mp.logical_order(7, 5, 1, 0, False, gm)) == list(range(35))


def test_arrival_order_pins():
    """Hand example and invariants of the arrival order (links of all ranks deliver side by side)."""
    # 3 ranks x 2 row blocks, rank 1 local: its blocks 2,3; then block 0 of ranks 2 and 0 (4, 0), then block 1 (5, 1)
    assert mp.arrival_rows(6, 3, 1) == [2, 3, 4, 0, 5, 1]
    assert mp.logical_order(6, 1, 3, 1, True, 1, True) == [2, 3, 4, 0, 5, 1]
    # falls back to the ring when a rank does not own whole row blocks, and to natural order without rotation
    assert mp.logical_order(5, 1, 2, 1, True, 1, True) == mp.logical_order(5, 1, 2, 1, True, 1, False)
    assert mp.logical_order(6, 1, 3, 1, False, 1, True) == [0, 1, 2, 3, 4, 5]
    for nbm, R, rank in [(32, 8, 5), (8, 8, 0), (12, 4, 3), (16, 2, 1)]:
        rows = mp.arrival_rows(nbm, R, rank)
        bpr = nbm // R
        assert sorted(rows) == list(range(nbm))
        assert all(r // bpr == rank for r in rows[:bpr])                      # the local shard first
        rest = rows[bpr:]
        assert [r % bpr for r in rest] == sorted(r % bpr for r in rest)        # block j of every rank before block j+1 of any
        for j in range(bpr):                                                   # inside a round: ring order from rank+1
            assert [r // bpr for r in rest[j * (R - 1):(j + 1) * (R - 1)]] == [(rank + q) % R for q in range(1, R)]
    # with grouping and the die swizzle it stays a permutation of all tiles
    sch = mp.tile_schedule(32, 14, 8, 5, True, 256, True, 4, True)
    assert sorted(sch) == list(range(32 * 14))


def test_rs_own_first_order():
    recs = mp.gemm_rs_schedule_records(1024, 512, 64, 4, 1, 256, 256, 128, 128, 8, True, False, 1, True)
    assert [r[1] for r in recs] == [1, 1, 2, 2, 3, 3, 0, 0]            # own segment (rank 1), then the ring 2, 3, 0
    order = mp.rs_consumer_order(1024, 512, 4, 1, 128, 128, True, True)
    assert order[:4] == [8, 9, 10, 11] and order[-4:] == [4, 5, 6, 7] and sorted(order) == list(range(32))
