"""The benchmark configurations at full size, in the launch configuration bench.py times."""
import numpy as np
import pytest
import torch

from conftest import set_flags
import oracle
import workloads
from test_gpu_parity import _check, _dev, _run_full

pytestmark = pytest.mark.gpu


def test_config3_full_oracle():
    print("config 3", flush=True)
    errs = _run_full(workloads.config(3))
    print(errs)


def test_config5_sampled_rows():
    """Config 5 is 10 TFLOP of fp64 work for the oracle; because rows do not interact, a sample of
    query rows (O, dQ) and key rows (dK, dV) is evaluated exactly instead: sequence ends, tile
    edges, and random rows of every sequence."""
    import paper_2508_04711_amd as lib
    w = workloads.config(5)
    vals = workloads.values(w)
    dev = _dev(vals)
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    outs = {}
    for odt in (torch.bfloat16, torch.float32):  # as bench.py runs it, and the accumulators unrounded
        o = lib.hstu_jagged_attn_fwd(dev["q"], dev["k"], dev["v"], off, w.max_len, w.alpha, True, out_dtype=odt)
        outs[odt] = (o,) + tuple(lib.hstu_jagged_attn_bwd(dev["q"], dev["k"], dev["v"], dev["d_o"], off, w.max_len,
                                                          w.alpha, True, out_dtype=odt))
    torch.cuda.synchronize()
    print("config 5 gpu done", flush=True)
    rng = np.random.default_rng(5)
    sel = []
    for b, L in enumerate(w.lengths):
        s = int(off_np[b])
        local = [0, 1, 127, 128, 129, L - 1, L - 2, L - 128, L - 129] + [int(x) for x in rng.integers(0, L, size=7)]
        sel += [s + x for x in local if 0 <= x < L]
    sel = sorted(set(sel))
    f64 = {k: workloads.to_f64(v) for k, v in vals.items()}
    want = oracle.rows(f64["q"], f64["k"], f64["v"], f64["d_o"], off_np, w.max_len, w.alpha, True, sel)
    print("config 5 oracle done", flush=True)
    # fp32 outputs: the stated bar; bf16 outputs: plus the storage rounding of the exact value
    for odt, got4 in outs.items():
        for name, got, ref in zip(("o", "dq", "dk", "dv"), got4, want):
            _check(name, got[sel], ref, "bf16", "config 5")
            # properties that hold at any size: finite everywhere
            assert torch.isfinite(got.float()).all()


def test_config5_with_timestamp_bias_sampled_rows():
    """bench.py's cfg5_bias workload (config 5 with sorted event timestamps, 64 buckets, four
    groups per octave) at full size: sampled query and key rows against the bias oracle.  The
    table gradient is a sum over every pair and cannot be sampled; it is checked against the
    full oracle at the sizes of tests/test_gpu_bias.py and here only for being finite."""
    import paper_2508_04711_amd as lib
    w = workloads.config(5)
    vals = workloads.values(w)
    dev = _dev(vals)
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    ts_np, tab_np = workloads.timestamps(w, "events", 0), workloads.bias_table(64, 0, 1.0)
    ts, tab = torch.from_numpy(ts_np).cuda(), torch.from_numpy(tab_np).cuda()
    outs = {}
    for odt in (torch.bfloat16, torch.float32):
        o = lib.hstu_jagged_attn_bias_fwd(dev["q"], dev["k"], dev["v"], off, ts, tab, 2, w.max_len, w.alpha, True,
                                          out_dtype=odt)
        outs[odt] = (o,) + tuple(lib.hstu_jagged_attn_bias_bwd(dev["q"], dev["k"], dev["v"], dev["d_o"], off, ts, tab,
                                                               2, w.max_len, w.alpha, True, out_dtype=odt))
    torch.cuda.synchronize()
    print("config 5 with bias: gpu done", flush=True)
    rng = np.random.default_rng(6)
    sel = []
    for b, L in enumerate(w.lengths):
        s = int(off_np[b])
        local = [0, 1, 127, 128, L - 1, L - 129] + [int(x) for x in rng.integers(0, L, size=4)]
        sel += [s + x for x in local if 0 <= x < L]
    sel = sorted(set(sel))
    f64 = {k: workloads.to_f64(v) for k, v in vals.items()}
    want = oracle.bias_rows(f64["q"], f64["k"], f64["v"], f64["d_o"], off_np, ts_np,
                            tab_np.astype(np.float64), 2, w.max_len, w.alpha, True, sel)
    print("config 5 with bias: oracle done", flush=True)
    for odt, got5 in outs.items():
        for name, got, ref in zip(("o", "dq", "dk", "dv"), got5, want):
            _check(name, got[sel], ref, "bf16", "config 5 with bias")
        for t in got5:
            assert torch.isfinite(t.float()).all()
        assert (got5[4] != 0).any()


@pytest.mark.parametrize("with_bias", [False, True])
def test_one_very_long_sequence(with_bias):
    """70 000 rows in one sequence (beyond any benchmark configuration): 1094 streamed tiles per
    pass, heavy query tiles cut along the keys, and with the bias 35 refills of the per-lane block
    table.  Sampled rows against the oracles."""
    import paper_2508_04711_amd as lib
    L = 70000
    w = workloads.custom("very_long", [L, 300], 2, 64, 64, L, dtype="bf16", seed=21)
    vals = workloads.values(w)
    dev = _dev(vals)
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    f64 = {k: workloads.to_f64(v) for k, v in vals.items()}
    rng = np.random.default_rng(7)
    sel = sorted(set([0, 1, 63, 64, 4095, 4096, L - 1, L - 129, L, L + 299] + [int(x) for x in rng.integers(0, L, size=10)]))
    if with_bias:
        ts_np, tab_np = workloads.timestamps(w, "events", 3), workloads.bias_table(96, 3)
        ts, tab = torch.from_numpy(ts_np).cuda(), torch.from_numpy(tab_np).cuda()
        o = lib.hstu_jagged_attn_bias_fwd(dev["q"], dev["k"], dev["v"], off, ts, tab, 2, w.max_len, w.alpha, True,
                                          out_dtype=torch.float32)
        dq, dk, dv, dw = lib.hstu_jagged_attn_bias_bwd(dev["q"], dev["k"], dev["v"], dev["d_o"], off, ts, tab, 2,
                                                       w.max_len, w.alpha, True, out_dtype=torch.float32)
        torch.cuda.synchronize()
        assert torch.isfinite(dw).all()
        want = oracle.bias_rows(f64["q"], f64["k"], f64["v"], f64["d_o"], off_np, ts_np,
                                tab_np.astype(np.float64), 2, w.max_len, w.alpha, True, sel)
    else:
        o = lib.hstu_jagged_attn_fwd(dev["q"], dev["k"], dev["v"], off, w.max_len, w.alpha, True,
                                     out_dtype=torch.float32)
        dq, dk, dv = lib.hstu_jagged_attn_bwd(dev["q"], dev["k"], dev["v"], dev["d_o"], off, w.max_len, w.alpha,
                                              True, out_dtype=torch.float32)
        torch.cuda.synchronize()
        want = oracle.rows(f64["q"], f64["k"], f64["v"], f64["d_o"], off_np, w.max_len, w.alpha, True, sel)
    print("very long: gpu and oracle done", with_bias, flush=True)
    # the bar is relative to the RMS of the whole tensor; the sampled rows' RMS stands in for it,
    # taken over the long sequence's rows (the short one's outputs are far larger: few terms / N)
    for name, got, ref in zip(("o", "dq", "dk", "dv"), (o, dq, dk, dv), want):
        g = got[sel].double().cpu().numpy()
        err = np.abs(g - ref)
        for rows_idx in ([i for i, r in enumerate(sel) if r < L], [i for i, r in enumerate(sel) if r >= L]):
            rms = float(np.sqrt((ref[rows_idx] ** 2).mean()))
            assert err[rows_idx].max() <= 2e-2 * rms, (name, float(err[rows_idx].max() / rms))
    for t in (o, dq, dk, dv):
        assert torch.isfinite(t).all()


@pytest.mark.parametrize("with_bias", [False, True])
def test_tensors_beyond_four_gib(with_bias):
    """1024 sequences of 4200 rows, H = 4, d = 128: every tensor is 4.4e9 bytes, so byte offsets
    of the rows of the last 25 sequences do not fit 32 bits.  The inputs are drawn on the device;
    the oracle gets the sequences the sampled rows lie in (rows of different sequences do not
    interact): the first, the one that contains byte offset 2^32, its successor, and the last."""
    import paper_2508_04711_amd as lib
    L, B, H, d = 4200, 1024, 4, 128
    w = workloads.custom("beyond_4gib", [L] * B, H, d, d, L, dtype="bf16", seed=31)
    assert w.total_rows * H * d * 2 > 2 ** 32
    dev = workloads.device_values(w)
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    straddle = (2 ** 32 // (H * d * 2)) // L
    seqs = [0, straddle, straddle + 1, B - 1]
    assert int(off_np[straddle]) * H * d * 2 < 2 ** 32 < int(off_np[straddle + 1]) * H * d * 2
    print("beyond 4 GiB: inputs drawn", with_bias, flush=True)
    ts = tab = None
    if with_bias:
        ts_np, tab_np = workloads.timestamps(w, "events", 5), workloads.bias_table(64, 5)
        ts, tab = torch.from_numpy(ts_np).cuda(), torch.from_numpy(tab_np).cuda()

    def run(odt):
        if with_bias:
            o = lib.hstu_jagged_attn_bias_fwd(dev["q"], dev["k"], dev["v"], off, ts, tab, 2, w.max_len, w.alpha, True,
                                              out_dtype=odt)
            dq, dk, dv, dw = lib.hstu_jagged_attn_bias_bwd(dev["q"], dev["k"], dev["v"], dev["d_o"], off, ts, tab, 2,
                                                           w.max_len, w.alpha, True, out_dtype=odt)
            torch.cuda.synchronize()
            assert torch.isfinite(dw).all() and (dw != 0).any()
        else:
            o = lib.hstu_jagged_attn_fwd(dev["q"], dev["k"], dev["v"], off, w.max_len, w.alpha, True, out_dtype=odt)
            dq, dk, dv = lib.hstu_jagged_attn_bwd(dev["q"], dev["k"], dev["v"], dev["d_o"], off, w.max_len, w.alpha,
                                                  True, out_dtype=odt)
            torch.cuda.synchronize()
        return o, dq, dk, dv
    # the sub-problem of the chosen sequences, with offsets of its own
    rows = np.concatenate([np.arange(off_np[b], off_np[b + 1]) for b in seqs])
    rows_t = torch.from_numpy(rows).cuda()
    sub = {k: workloads.to_f64(v[rows_t]) for k, v in dev.items()}
    sub_off = (np.arange(len(seqs) + 1) * L).astype(np.int32)
    rng = np.random.default_rng(9)
    local = sorted(set([0, 1, 63, 64, 127, 128, L - 1, L - 2, L - 65] + [int(x) for x in rng.integers(0, L, size=6)]))
    sel = [i * L + x for i in range(len(seqs)) for x in local]
    if with_bias:
        want = oracle.bias_rows(sub["q"], sub["k"], sub["v"], sub["d_o"], sub_off, ts_np[rows],
                                tab_np.astype(np.float64), 2, w.max_len, w.alpha, True, sel)
    else:
        want = oracle.rows(sub["q"], sub["k"], sub["v"], sub["d_o"], sub_off, w.max_len, w.alpha, True, sel)
    print("beyond 4 GiB: oracle done", flush=True)
    glob = torch.from_numpy(rows[sel]).cuda()
    for odt in (torch.bfloat16, torch.float32):  # fp32: the stated bar; bf16: plus the storage rounding
        outs = run(odt)
        for name, got, ref in zip(("o", "dq", "dk", "dv"), outs, want):
            _check(name, got[glob], ref, "bf16", "beyond 4 GiB")
        # every sequence has the same shape, so outputs beyond 4 GiB are as large as those before it
        for t in outs:
            head, tail = t[:L * 8].float(), t[-L * 8:].float()
            assert torch.isfinite(tail).all()
            assert 0.8 < float(tail.pow(2).mean().sqrt() / head.pow(2).mean().sqrt()) < 1.25
        del outs


@pytest.mark.parametrize("mode", ["plain", "bias", "packed"])
def test_large_batch_of_short_sequences(mode, monkeypatch):
    """4096 sequences of 32..256 rows, H = 4, d = 128: a batch large enough for the natural item
    order and for the dK/dV workgroups that walk over items (per-sequence tiles with and without
    the bias, packed tiles).  Sampled rows of a few sequences against the oracle on those
    sequences alone (rows of different sequences do not interact)."""
    import paper_2508_04711_amd as lib
    if mode == "packed":
        set_flags(monkeypatch, add="PACK_SHORT")
    else:
        set_flags(monkeypatch, add="NO_PACK")
    rng = np.random.default_rng(17)
    lengths = [int(x) for x in rng.integers(32, 257, size=4096)]
    w = workloads.custom("large_batch", lengths, 4, 128, 128, 256, dtype="bf16", seed=41)
    vals = workloads.values(w)
    dev = _dev(vals)
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    print("large batch", mode, w.total_rows, flush=True)
    ts = tab = None
    if mode == "bias":
        ts_np, tab_np = workloads.timestamps(w, "events", 6), workloads.bias_table(48, 6)
        ts, tab = torch.from_numpy(ts_np).cuda(), torch.from_numpy(tab_np).cuda()

    def run(odt):
        if mode == "bias":
            o = lib.hstu_jagged_attn_bias_fwd(dev["q"], dev["k"], dev["v"], off, ts, tab, 1, w.max_len, w.alpha, True,
                                              out_dtype=odt)
            dq, dk, dv, dw = lib.hstu_jagged_attn_bias_bwd(dev["q"], dev["k"], dev["v"], dev["d_o"], off, ts, tab, 1,
                                                           w.max_len, w.alpha, True, out_dtype=odt)
            assert torch.isfinite(dw).all() and (dw != 0).any()
        else:
            o = lib.hstu_jagged_attn_fwd(dev["q"], dev["k"], dev["v"], off, w.max_len, w.alpha, True, out_dtype=odt)
            dq, dk, dv = lib.hstu_jagged_attn_bwd(dev["q"], dev["k"], dev["v"], dev["d_o"], off, w.max_len, w.alpha,
                                                  True, out_dtype=odt)
        torch.cuda.synchronize()
        return o, dq, dk, dv
    seqs = [0, 1, 255, 256, 2047, 3000, 4094, 4095]
    rows = np.concatenate([np.arange(off_np[b], off_np[b + 1]) for b in seqs])
    sub = {k: workloads.to_f64(v[torch.from_numpy(rows)]) for k, v in vals.items()}
    sub_off = np.concatenate([[0], np.cumsum([lengths[b] for b in seqs])]).astype(np.int32)
    sel = np.arange(len(rows))
    if mode == "bias":
        want = oracle.bias_rows(sub["q"], sub["k"], sub["v"], sub["d_o"], sub_off, ts_np[rows],
                                tab_np.astype(np.float64), 1, w.max_len, w.alpha, True, sel)
    else:
        want = oracle.rows(sub["q"], sub["k"], sub["v"], sub["d_o"], sub_off, w.max_len, w.alpha, True, sel)
    glob = torch.from_numpy(rows).cuda()
    # the stated bar on the fp32 accumulators (measured 1.1e-2 .. 1.3e-2), the storage rounding on top for bf16
    for odt in (torch.float32, torch.bfloat16):
        outs = run(odt)
        for name, got, ref in zip(("o", "dq", "dk", "dv"), outs, want):
            _check(name, got[glob], ref, "bf16", "large batch %s" % mode)
        for t in outs:
            assert torch.isfinite(t.float()).all()


@pytest.mark.parametrize("H,B", [(1, 16384), (2, 8192), (3, 8192)])
def test_large_batch_head_counts(H, B, monkeypatch):
    """Large batches with other head counts, per-sequence tiles: 1 and 2 heads take the map that
    gives every XCD one head and one contiguous part of the item list (8 and 4 parts), 3 heads the
    plain map with the dK/dV workgroups walking over the sorted list.  Sampled sequences against
    the oracle on those sequences alone."""
    import paper_2508_04711_amd as lib
    set_flags(monkeypatch, add="NO_PACK")
    rng = np.random.default_rng(23 + H)
    lengths = [int(x) for x in rng.integers(32, 257, size=B)]
    w = workloads.custom("large_batch_h%d" % H, lengths, H, 128, 128, 256, dtype="bf16", seed=50 + H)
    dev = workloads.device_values(w)
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    print("large batch heads", H, B, w.total_rows, flush=True)
    seqs = [0, 1, B // 8 - 1, B // 8, B // 2, B - 2, B - 1]
    rows = np.concatenate([np.arange(off_np[b], off_np[b + 1]) for b in seqs])
    rows_t = torch.from_numpy(rows).cuda()
    sub = {k: workloads.to_f64(v[rows_t]) for k, v in dev.items()}
    sub_off = np.concatenate([[0], np.cumsum([lengths[b] for b in seqs])]).astype(np.int32)
    want = oracle.rows(sub["q"], sub["k"], sub["v"], sub["d_o"], sub_off, w.max_len, w.alpha, True,
                       np.arange(len(rows)))
    for odt in (torch.float32, torch.bfloat16):  # fp32: the stated bar; bf16: plus the storage rounding
        o = lib.hstu_jagged_attn_fwd(dev["q"], dev["k"], dev["v"], off, w.max_len, w.alpha, True, out_dtype=odt)
        dq, dk, dv = lib.hstu_jagged_attn_bwd(dev["q"], dev["k"], dev["v"], dev["d_o"], off, w.max_len, w.alpha, True,
                                              out_dtype=odt)
        torch.cuda.synchronize()
        for name, got, ref in zip(("o", "dq", "dk", "dv"), (o, dq, dk, dv), want):
            _check(name, got[rows_t], ref, "bf16", "large batch, %d heads" % H)
        # every row was written: the outputs of all sequences are of one scale
        for t in (o, dq, dk, dv):
            assert torch.isfinite(t.float()).all()
            a = t[: w.total_rows // 2].float().pow(2).mean().sqrt()
            b = t[w.total_rows // 2:].float().pow(2).mean().sqrt()
            assert 0.8 < float(a / b) < 1.25
