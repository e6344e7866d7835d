"""The synthetic workloads are pinned: lengths, totals and flop counts."""
import numpy as np

import workloads


def test_config_lengths_and_totals():
    totals = {1: 147, 2: 17286, 3: 37117, 4: 66088, 5: 96016}
    for cfg, T in totals.items():
        w = workloads.config(cfg)
        assert w.total_rows == T
        off = w.seq_offsets()
        assert off.dtype == np.int32 and off[0] == 0 and off[-1] == T
    assert workloads.config(1).lengths == (55, 41, 33, 18)
    assert all(l % 8 == 0 for l in workloads.config(4).lengths)
    assert workloads.config(3).pairs_per_head == 52957147
    assert workloads.config(5).pairs_per_head == 698506850


def test_large_batches_are_pinned():
    short, mid = workloads.large_batch("short"), workloads.large_batch("mid")
    assert (short.batch, short.total_rows, short.pairs_per_head) == (8192, 328154, 7548970)
    assert (mid.batch, mid.total_rows, mid.pairs_per_head) == (1536, 693773, 162709638)
    assert min(short.lengths) == 16 and max(short.lengths) == 64 == short.max_len
    assert min(mid.lengths) >= 300 and max(mid.lengths) <= 600 == mid.max_len


def test_flop_counts():
    w = workloads.config(3)
    f = w.flops()
    assert abs(f["fwd"] / 1e9 - 108.5) < 0.1 and abs(f["bwd"] / 1e9 - 271.1) < 0.1


def test_values_are_seeded_and_rounded_once():
    w = workloads.config(1)
    a, b = workloads.values(w), workloads.values(w)
    for name in ("q", "k", "v", "d_o"):
        assert a[name].dtype.is_floating_point and (a[name] == b[name]).all()
    w2 = workloads.custom("t", [3, 4], 2, 32, 32, 8, dtype="bf16")
    x = workloads.values(w2)["q"]
    assert np.array_equal(workloads.to_f64(x), x.float().double().numpy())


def test_timestamps_and_tables_are_seeded_and_shaped():
    w = workloads.custom("t", [40, 0, 7, 300], 1, 32, 32, 300)
    off = w.seq_offsets()
    for kind in ("events", "shuffled", "equal", "wide"):
        ts = workloads.timestamps(w, kind, 3)
        assert ts.dtype == np.int32 and ts.shape == (w.total_rows,)
        assert np.array_equal(ts, workloads.timestamps(w, kind, 3))          # seeded
        assert not np.array_equal(ts, workloads.timestamps(w, kind, 4)) or kind == "never"
        for b in range(w.batch):
            seg = ts[off[b]:off[b + 1]].astype(np.int64)
            if kind in ("events", "wide"):
                assert (np.diff(seg) >= 0).all()                               # a history is sorted
            if kind == "equal":
                assert (seg == seg[:1]).all()
    sh = workloads.timestamps(w, "shuffled", 3).astype(np.int64)
    assert (np.diff(sh[off[3]:off[4]]) < 0).any()                              # not sorted
    span = workloads.timestamps(w, "wide", 3).astype(np.int64)
    assert span.max() - span.min() > 2 ** 31                                   # differences beyond int32
    tab = workloads.bias_table(24, 1, 0.5)
    assert tab.dtype == np.float32 and tab.shape == (24,) and np.array_equal(tab, workloads.bias_table(24, 1, 0.5))
