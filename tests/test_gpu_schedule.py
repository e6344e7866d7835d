"""The device-built schedule (tile table) against a re-derivation in Python: integer work, exact.

Jagged addressing must be bit-exact: every tile's rows, positions and streamed segments must be
exactly those the offsets imply, every owner row must belong to exactly one tile, tiles wholly
above the diagonal must be absent, and heavy tiles must come first.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _side(L, cp, rank):
    """Segments [(pos, len)] of one side of a sequence (rank < 0: the whole sequence)."""
    if rank < 0:
        return [(0, L)]
    c = -(-L // (2 * cp))
    segs = []
    for m in (rank, 2 * cp - 1 - rank):
        lo, hi = min(m * c, L), min((m + 1) * c, L)
        segs.append((lo, hi - lo))
    if segs[1][1] > 0 and segs[1][0] == segs[0][0] + segs[0][1]:
        segs = [(segs[0][0], segs[0][1] + segs[1][1])]
    return [s for i, s in enumerate(segs) if s[1] > 0 or i == 0]


def _expected_items(lengths, tile, causal, side, cp=1, owner_rank=-1, streamed_rank=-1):
    items = []
    obase = sbase = 0
    off = 0
    for L in lengths:
        osegs, ssegs = _side(L, cp, owner_rank), _side(L, cp, streamed_rank)
        ob = off if owner_rank < 0 else obase
        sb = off if streamed_rank < 0 else sbase
        orow = ob
        for (opos, olen) in osegs:
            for t in range(0, olen, tile):
                nrows = min(tile, olen - t)
                pos0 = opos + t
                segs, cost, srow = [], 0, sb
                for (spos, slen) in ssegs:
                    if not causal:
                        vis = slen
                    elif side == 0:
                        vis = min(max(pos0 + nrows - spos, 0), slen)
                    else:
                        vis = slen - min(max(pos0 - spos, 0), slen)
                    if vis > 0:
                        segs.append((srow, slen, spos))
                        cost += (vis + 31) // 32
                    srow += slen
                segs += [(0, 0, 0)] * (2 - len(segs))
                nseg = sum(1 for s in segs if s[1] > 0)
                items.append((orow + t, nrows, pos0, nseg, segs[0][0], segs[1][0], segs[0][1],
                              segs[1][1], segs[0][2], segs[1][2], cost, 0))
            orow += olen
        obase += sum(s[1] for s in osegs)
        sbase += sum(s[1] for s in ssegs)
        off += L
    return items


CASES = [
    ([55, 41, 33, 18], True),
    ([1, 0, 129, 128, 127, 0, 700, 3], True),
    ([300, 5, 260], False),
    (list(np.random.default_rng(5).integers(0, 600, size=70)), True),
    # batches larger than one pass of the schedule kernel's 1024 threads, kept in LDS ...
    (list(np.random.default_rng(6).integers(0, 300, size=1500)), True),
    (list(np.random.default_rng(7).integers(32, 257, size=4096)), True),
    # ... and larger than what it keeps in LDS (per-sequence bases in the workspace)
    (list(np.random.default_rng(8).integers(0, 40, size=7000)), True),
]


@pytest.mark.parametrize("side", [0, 1])
@pytest.mark.parametrize("lengths,causal", CASES)
def test_full_attention_schedule(lengths, causal, side):
    import paper_2508_04711_amd as lib
    lengths = [int(x) for x in lengths]
    T = sum(lengths)
    off = torch.tensor(np.concatenate([[0], np.cumsum(lengths)]), dtype=torch.int32, device="cuda")
    tile = lib.hstu_schedule_tile_rows(0, 128, 128, side, T, 2, len(lengths))
    got = lib.hstu_debug_dump_schedule(off, T, 2, 128, 128, causal, 0, side, max_len=max(lengths + [1]))
    want = _expected_items(lengths, tile, causal, side)
    assert sorted(map(tuple, got.tolist())) == sorted(want)
    costs = got[:, 10].astype(np.int64)
    # Heavy tiles first, unless even the heaviest tile is small against what one of the 512
    # workgroup slots gets in total: then the library may keep the natural order.  It decides from
    # bounds (max_len for the heaviest tile, the mean length for the total), which this condition,
    # from the actual costs, implies: a cost of c means more than 32 (c - 1) streamed rows, and a
    # tile's pairs are at most 32 x tile x cost.
    if (costs.max() - 1) * 8 * 512 > costs.sum() * 2:
        assert np.all(costs[:-1] >= costs[1:]), "heavy tiles first"
    covered = np.zeros(T, dtype=np.int64)
    for it in got:
        covered[it[0]:it[0] + it[1]] += 1
    assert np.all(covered == 1), "every row in exactly one tile"


@pytest.mark.parametrize("side", [0, 1])
@pytest.mark.parametrize("cp,q_rank,kv_rank", [(2, 0, 1), (2, 1, 0), (4, 3, -1), (4, 0, 0), (3, 1, 2), (1, 0, 0)])
def test_context_parallel_schedule(cp, q_rank, kv_rank, side):
    import oracle
    import paper_2508_04711_amd as lib
    lengths = [16, 5, 0, 233, 1, 400, 64, 777]
    T = sum(lengths)
    off_np = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    off = torch.from_numpy(off_np).cuda()
    nq = len(oracle.cp_global_rows(off_np, cp, q_rank))
    nk = len(oracle.cp_global_rows(off_np, cp, kv_rank))
    tile = lib.hstu_schedule_tile_rows(0, 64, 64, side)
    got = lib.hstu_debug_dump_schedule(off, T, 2, 64, 64, True, 0, side, cp=(cp, q_rank, kv_rank, nq, nk))
    owner, streamed = (q_rank, kv_rank) if side == 0 else (kv_rank, q_rank)
    want = _expected_items(lengths, tile, True, side, cp, owner, streamed)
    assert sorted(map(tuple, got.tolist())) == sorted(want)
    covered = np.zeros(nq if side == 0 else nk, dtype=np.int64)
    for it in got:
        covered[it[0]:it[0] + it[1]] += 1
    assert np.all(covered == 1)


def test_inconsistent_offsets_never_leave_the_declared_rows():
    # offsets that overshoot the declared total: tiles are clipped to the declared rows
    import paper_2508_04711_amd as lib
    off = torch.tensor([0, 100, 5000], dtype=torch.int32, device="cuda")
    got = lib.hstu_debug_dump_schedule(off, 300, 1, 64, 64, True, 0, 0)
    for it in got:
        assert 0 <= it[0] and it[0] + it[1] <= 300
        for g in range(it[3]):
            assert 0 <= it[4 + g] and it[4 + g] + it[6 + g] <= 300


@pytest.mark.parametrize("cp", [None, (2, 1, -1)])
def test_heavy_query_tiles_are_cut_along_the_keys(cp):
    """Few query tiles, long sequences: heavy tiles appear as several items, each covering a run of
    whole 64-key tiles, which together cover the tile's visible keys exactly once."""
    import oracle
    import paper_2508_04711_amd as lib
    lengths = [9000, 5000, 700, 64]
    T = sum(lengths)
    off_np = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    off = torch.from_numpy(off_np).cuda()
    if cp is None:
        got = lib.hstu_debug_dump_schedule(off, T, 1, 128, 128, True, 0, 0, max_len=9000)
    else:
        nq = len(oracle.cp_global_rows(off_np, cp[0], cp[1]))
        got = lib.hstu_debug_dump_schedule(off, T, 1, 128, 128, True, 0, 0,
                                           cp=(cp[0], cp[1], cp[2], nq, T), max_len=9000)
    parts = got[got[:, 11] > 0]
    whole = got[got[:, 11] == 0]
    assert len(parts) > 0, "the long sequences must produce split tiles"
    assert len(set(parts[:, 11].tolist())) == len(parts), "every part has a partial slot of its own"
    by_tile = {}
    for it in parts:
        by_tile.setdefault((int(it[0]), int(it[1]), int(it[2])), []).append(it)
    for (row0, nrows, pos0), its in by_tile.items():
        assert len(its) >= 2
        slots = sorted(int(it[11]) for it in its)
        assert slots == list(range(slots[0], slots[0] + len(its))), "consecutive slots, summed in order"
        # visible key positions of this query tile: 0 .. pos0 + nrows - 1 (causal, whole sequence streamed)
        seen = np.zeros(pos0 + nrows, dtype=np.int64)
        for it in its:
            for g in range(int(it[3])):
                spos, slen = int(it[8 + g]), int(it[6 + g])
                assert spos % 64 == 0 or cp is not None
                hi = min(spos + slen, pos0 + nrows)
                seen[spos:hi] += 1
        assert np.all(seen == 1), (row0, seen.min(), seen.max())
    # a tile is either whole or in parts, never both
    whole_tiles = {(int(it[0]), int(it[1])) for it in whole}
    assert not (whole_tiles & {(k[0], k[1]) for k in by_tile})
