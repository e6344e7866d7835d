"""Attention with the timestamp bias (forward, dQ/dK/dV and the gradient of the bucket table)
on the GPU against oracle/hstu_oracle_bias.c, through the C ABI.

Tolerances: o, dq, dk, dv as for the calls without bias (max abs error <= 2e-2 x RMS of the exact
tensor, plus half a bf16 ulp when the output is bf16).  The table gradient is a sum of fp32 dS
values that are never rounded to bf16, accumulated in fp32: <= 2e-3 x RMS over the buckets."""
import numpy as np
import pytest
import torch

from conftest import set_flags
import oracle
import workloads
from test_gpu_parity import _check, _dev

pytestmark = pytest.mark.gpu


def _run(w, kind, nb, f, causal=True, wscale=1.0, out_dtype=torch.float32, seed=0, check=None):
    """check(name, got, want, tag): replaces the standard bar for o, dq, dk, dv (batches of very short
    sequences, whose outputs are sums of a handful of terms, state their own)."""
    import paper_2508_04711_amd as lib
    if check is None:
        check = lambda name, got, ref, tag: _check(name, got, ref, w.dtype, tag)
    vals = workloads.values(w)
    dev = _dev(vals)
    f64 = {k: workloads.to_f64(v) for k, v in vals.items()}
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    ts_np = workloads.timestamps(w, kind, seed)
    tab_np = workloads.bias_table(nb, seed, wscale)
    ts, tab = torch.from_numpy(ts_np).cuda(), torch.from_numpy(tab_np).cuda()
    want = oracle.bias_attention(f64["q"], f64["k"], f64["v"], f64["d_o"], off_np, ts_np,
                                 tab_np.astype(np.float64), f, w.max_len, w.alpha, causal)
    tag = "%s/%s/nb%d/f%d/%s" % (w.name, kind, nb, f, "causal" if causal else "full")
    print("bias", tag, flush=True)
    o = lib.hstu_jagged_attn_bias_fwd(dev["q"], dev["k"], dev["v"], off, ts, tab, f, w.max_len, w.alpha,
                                      causal, out_dtype=out_dtype)
    torch.cuda.synchronize()
    check("o", o, want[0], tag)
    dq, dk, dv, dw = lib.hstu_jagged_attn_bias_bwd(dev["q"], dev["k"], dev["v"], dev["d_o"], off, ts, tab,
                                                   f, w.max_len, w.alpha, causal, out_dtype=out_dtype)
    torch.cuda.synchronize()
    check("dq", dq, want[1], tag)
    check("dk", dk, want[2], tag)
    check("dv", dv, want[3], tag)
    got = dw.double().cpu().numpy()
    assert np.isfinite(got).all()
    rms = float(np.sqrt(np.mean(want[4] ** 2)))
    err = float(np.abs(got - want[4]).max())
    print("   dw: max|err|/rms = %.2e" % (err / max(rms, 1e-300)), flush=True)
    # fp32 inputs: a bucket's entry is an fp32 sum of up to ~1e5 terms of either sign, added in an
    # order the atomics decide; its rounding error grows with the sum of the magnitudes, not with
    # the (cancelling) result: 1e-4 x RMS leaves an order of magnitude over the ~1e-5 measured
    bar = 2e-3 if w.dtype == "bf16" else 1e-4
    assert err <= bar * rms + 1e-30, "%s dw: max|err|/rms = %.3e" % (tag, err / max(rms, 1e-300))
    # buckets no pair falls into stay exactly zero
    assert (got[want[4] == 0.0] == 0.0).all()
    return dw


LENGTHS = [700, 130, 1, 519, 0, 64, 33]


@pytest.mark.parametrize("kind", ["events", "shuffled", "equal", "wide"])
@pytest.mark.parametrize("d", [32, 64, 128])
def test_bias_matches_oracle(kind, d):
    w = workloads.custom("bias_small", LENGTHS, 2, d, d, 700, dtype="bf16", seed=20 + d)
    _run(w, kind, nb=40, f=2, causal=True, seed=d)


@pytest.mark.parametrize("kind", ["events", "shuffled"])
def test_bias_one_wave_dkdv_kernel(kind, monkeypatch):
    """d = 128 with per-sequence tiles runs the dk/dv kernel with two waves per 32 keys (above); the
    one-wave kernel, which packed tiles and large batches run with the bias, is selected by its flag."""
    set_flags(monkeypatch, add="DKDV_ONE_WAVE")
    w = workloads.custom("bias_one_wave", LENGTHS, 2, 128, 128, 700, dtype="bf16", seed=31)
    _run(w, kind, nb=40, f=2, causal=True, seed=7)


@pytest.mark.parametrize("nb,f", [(1, 0), (7, 0), (33, 1), (512, 4), (300, 8)])
def test_bias_bucket_shapes(nb, f):
    w = workloads.custom("bias_buckets", [300, 257, 90], 2, 64, 64, 300, dtype="bf16", seed=5)
    _run(w, "events", nb=nb, f=f, seed=nb)


@pytest.mark.parametrize("dqk,dv", [(128, 64), (64, 128), (32, 128), (128, 32), (64, 32), (32, 64)])
def test_bias_unequal_head_dimensions(dqk, dv):
    w = workloads.custom("bias_dims", [300, 129, 75], 2, dqk, dv, 300, dtype="bf16", seed=dqk + dv)
    _run(w, "events", nb=40, f=2, seed=dqk)


def test_bias_non_causal_and_bf16_outputs():
    w = workloads.custom("bias_full", [260, 75, 130], 3, 64, 64, 260, dtype="bf16", seed=6)
    _run(w, "events", nb=24, f=1, causal=False, seed=1)
    _run(w, "shuffled", nb=24, f=1, causal=False, seed=2)
    _run(w, "events", nb=24, f=1, causal=True, out_dtype=torch.bfloat16, seed=3)


def test_bias_long_sequence_with_key_split_and_wide_tiles():
    """One long sequence: the forward and dQ passes cut their heavy query tiles along the keys,
    and most blocks are far from the diagonal (one bucket per block)."""
    w = workloads.custom("bias_long", [4700, 300], 1, 64, 64, 4700, dtype="bf16", seed=8)
    _run(w, "events", nb=64, f=2, seed=4)


def test_bias_many_short_sequences():
    """Mean length below the threshold of the form without a transposed copy of V."""
    rng = np.random.default_rng(3)
    lengths = [int(x) for x in rng.integers(1, 200, size=40)]
    w = workloads.custom("bias_short", lengths, 2, 128, 128, 200, dtype="bf16", seed=9)
    _run(w, "events", nb=48, f=2, seed=5)


def test_zero_table_equals_the_call_without_bias(monkeypatch):
    import paper_2508_04711_amd as lib
    set_flags(monkeypatch, add="NO_PACK")   # the calls with bias tile per sequence: so must the other
    w = workloads.custom("bias_zero", [700, 130, 519], 2, 64, 64, 700, dtype="bf16", seed=11)
    dev = _dev(workloads.values(w))
    off = torch.from_numpy(w.seq_offsets()).cuda()
    ts = torch.from_numpy(workloads.timestamps(w, "events", 1)).cuda()
    tab = torch.zeros(32, dtype=torch.float32, device="cuda")
    o0 = lib.hstu_jagged_attn_fwd(dev["q"], dev["k"], dev["v"], off, w.max_len, w.alpha, True)
    o1 = lib.hstu_jagged_attn_bias_fwd(dev["q"], dev["k"], dev["v"], off, ts, tab, 2, w.max_len, w.alpha, True)
    g0 = lib.hstu_jagged_attn_bwd(dev["q"], dev["k"], dev["v"], dev["d_o"], off, w.max_len, w.alpha, True)
    g1 = lib.hstu_jagged_attn_bias_bwd(dev["q"], dev["k"], dev["v"], dev["d_o"], off, ts, tab, 2, w.max_len,
                                       w.alpha, True)
    torch.cuda.synchronize()
    # adding 0.0 to the accumulator before the products changes no bit
    assert torch.equal(o0, o1)
    for a, b in zip(g0, g1[:3]):
        assert torch.equal(a, b)


def test_bias_argument_errors():
    import paper_2508_04711_amd as lib
    w = workloads.custom("bias_err", [64, 64], 1, 32, 32, 64, dtype="bf16", seed=1)
    dev = _dev(workloads.values(w))
    off = torch.from_numpy(w.seq_offsets()).cuda()
    ts = torch.from_numpy(workloads.timestamps(w, "events", 1)).cuda()
    tab = torch.zeros(8, dtype=torch.float32, device="cuda")
    with pytest.raises(lib.HstuError) as e:      # groups_log2 out of range
        lib.hstu_jagged_attn_bias_fwd(dev["q"], dev["k"], dev["v"], off, ts, tab, 9, 64, w.alpha, True)
    assert e.value.status == -2
    big = torch.zeros(513, dtype=torch.float32, device="cuda")
    with pytest.raises(lib.HstuError) as e:      # too many buckets
        lib.hstu_jagged_attn_bias_fwd(dev["q"], dev["k"], dev["v"], off, ts, big, 2, 64, w.alpha, True)
    assert e.value.status == -2
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(lib.HstuError) as e:
        lib.hstu_jagged_attn_bias_fwd(dev["q"], dev["k"], dev["v"], off, ts, tab, 2, 64, w.alpha, True,
                                      workspace=small)
    assert e.value.status == -4
    with pytest.raises(ValueError):              # one timestamp per row
        lib.hstu_jagged_attn_bias_fwd(dev["q"], dev["k"], dev["v"], off, ts[:-1].contiguous(), tab, 2, 64,
                                      w.alpha, True)


def _check_dw(got, want, tag):
    g = got.double().cpu().numpy()
    rms = float(np.sqrt(np.mean(want ** 2)))
    err = float(np.abs(g - want).max())
    assert np.isfinite(g).all() and err <= 2e-3 * rms + 1e-30, "%s dw: max|err|/rms = %.3e" % (tag, err / max(rms, 1e-300))


@pytest.mark.parametrize("cp", [2, 3])
def test_context_parallel_partials_with_bias(cp):
    """Every rank's queries (local layout, with their timestamps) against all keys in one call,
    and against each rank's keys in turn with accumulation: outputs per rank equal the oracle's
    rows, key-side gradients and the table gradient add up over the ranks to the whole batch's."""
    import paper_2508_04711_amd as lib
    lengths = [520, 96, 1030, 8, 0, 333]
    w = workloads.custom("cp_bias", lengths, 2, 64, 64, 1030, dtype="bf16", seed=30 + cp)
    vals = workloads.values(w)
    dev = _dev(vals)
    f64 = {k: workloads.to_f64(v) for k, v in vals.items()}
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    T = w.total_rows
    ts_np, tab_np = workloads.timestamps(w, "events", cp), workloads.bias_table(40, cp)
    ts, tab = torch.from_numpy(ts_np).cuda(), torch.from_numpy(tab_np).cuda()
    want = oracle.bias_attention(f64["q"], f64["k"], f64["v"], f64["d_o"], off_np, ts_np,
                                 tab_np.astype(np.float64), 2, w.max_len, w.alpha, True)
    rows = [oracle.cp_global_rows(off_np, cp, r) for r in range(cp)]
    trow = [torch.from_numpy(r).cuda() for r in rows]
    f32 = dict(dtype=torch.float32, device="cuda")

    # (a) all keys in the global layout
    dk_sum, dv_sum = torch.zeros((T, 2, 64), **f32), torch.zeros((T, 2, 64), **f32)
    dw_sum = torch.zeros(40, **f32)
    for rq in range(cp):
        print("cp bias", cp, rq, "all keys", flush=True)
        # the rank's rows and their timestamps, moved by the reorder kernel in one launch
        ql, gl, tq = lib.hstu_cp_reorder([dev["q"], dev["d_o"], ts], off, T, cp, rq, len(rows[rq]))
        assert torch.equal(tq, ts[trow[rq]])
        o, dq, dk, dv, dw = lib.hstu_jagged_attn_cp_partial_bias(
            ql, dev["k"], dev["v"], gl, off, T, tq, ts, tab, 2, w.max_len, w.alpha, True, cp, rq, -1,
            out_dtype=torch.float32)
        torch.cuda.synchronize()
        _check("o", o, want[0][rows[rq]], "bf16", "cp%d q%d" % (cp, rq))
        _check("dq", dq, want[1][rows[rq]], "bf16", "cp%d q%d" % (cp, rq))
        dk_sum += dk; dv_sum += dv; dw_sum += dw
        # forward only: the same o, no gradient buffers needed
        o2 = lib.hstu_jagged_attn_cp_partial_bias(ql, dev["k"], dev["v"], None, off, T, tq, ts, tab, 2,
                                                  w.max_len, w.alpha, True, cp, rq, -1,
                                                  out_dtype=torch.float32)[0]
        assert torch.equal(o2, o)
    _check("dk", dk_sum, want[2], "bf16", "cp%d all keys" % cp)
    _check("dv", dv_sum, want[3], "bf16", "cp%d all keys" % cp)
    _check_dw(dw_sum, want[4], "cp%d all keys" % cp)

    # (b) one key rank at a time, everything accumulated
    dk_sum.zero_(); dv_sum.zero_()
    dw_acc = torch.zeros(40, **f32)
    for rq in range(cp):
        ql, gl, tq = dev["q"][trow[rq]].contiguous(), dev["d_o"][trow[rq]].contiguous(), ts[trow[rq]].contiguous()
        o_acc = torch.zeros((len(rows[rq]), 2, 64), **f32)
        dq_acc = torch.zeros_like(o_acc)
        for rk in range(cp):
            print("cp bias", cp, rq, rk, flush=True)
            kl, vl, tk = dev["k"][trow[rk]].contiguous(), dev["v"][trow[rk]].contiguous(), ts[trow[rk]].contiguous()
            dk_run = torch.zeros((len(rows[rk]), 2, 64), **f32)
            dv_run = torch.zeros_like(dk_run)
            lib.hstu_jagged_attn_cp_partial_bias(ql, kl, vl, gl, off, T, tq, tk, tab, 2, w.max_len, w.alpha,
                                                 True, cp, rq, rk, accumulate=True,
                                                 out=(o_acc, dq_acc, dk_run, dv_run, dw_acc))
            dk_sum[trow[rk]] += dk_run
            dv_sum[trow[rk]] += dv_run
        torch.cuda.synchronize()
        _check("o sum", o_acc, want[0][rows[rq]], "bf16", "cp%d q%d" % (cp, rq))
        _check("dq sum", dq_acc, want[1][rows[rq]], "bf16", "cp%d q%d" % (cp, rq))
    _check("dk sum", dk_sum, want[2], "bf16", "cp%d" % cp)
    _check("dv sum", dv_sum, want[3], "bf16", "cp%d" % cp)
    _check_dw(dw_acc, want[4], "cp%d pairs" % cp)


@pytest.mark.parametrize("cp", [1, 2, 4])
def test_ring_pass_with_bias(cp):
    """Every rank's ring pass with the bias: the parts' timestamps travel with their K and V; o and
    dq per rank equal the oracle's rows, the key-side gradients (added to travelling buffers) and
    the ranks' table gradients add up to the whole batch's."""
    import paper_2508_04711_amd as lib
    lengths = [160, 5, 233, 1, 0, 384, 77, 900]
    w = workloads.custom("ring_bias", lengths, 2, 64, 64, 900, dtype="bf16", seed=40 + cp)
    vals = workloads.values(w)
    dev = _dev(vals)
    f64 = {k: workloads.to_f64(v) for k, v in vals.items()}
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    T = w.total_rows
    ts_np, tab_np = workloads.timestamps(w, "events", cp), workloads.bias_table(48, cp)
    ts, tab = torch.from_numpy(ts_np).cuda(), torch.from_numpy(tab_np).cuda()
    want = oracle.bias_attention(f64["q"], f64["k"], f64["v"], f64["d_o"], off_np, ts_np,
                                 tab_np.astype(np.float64), 2, w.max_len, w.alpha, True)
    rows = [oracle.cp_global_rows(off_np, cp, r) for r in range(cp)]
    parts = [lib.hstu_cp_reorder([dev["k"], dev["v"], ts], off, T, cp, r, len(rows[r])) for r in range(cp)]
    kp, vp, tp = [p[0] for p in parts], [p[1] for p in parts], [p[2] for p in parts]
    f32 = dict(dtype=torch.float32, device="cuda")
    dks = [torch.zeros((len(rows[r]), 2, 64), **f32) for r in range(cp)]
    dvs = [torch.zeros((len(rows[r]), 2, 64), **f32) for r in range(cp)]
    dw_sum = torch.zeros(48, **f32)
    for rq in range(cp):
        print("ring with bias", cp, rq, flush=True)
        ql, gl, tq = lib.hstu_cp_reorder([dev["q"], dev["d_o"], ts], off, T, cp, rq, len(rows[rq]))
        nq = len(rows[rq])
        o, dq = torch.empty((nq, 2, 64), **f32), torch.empty((nq, 2, 64), **f32)
        dw = torch.full((48,), float("nan"), **f32)          # overwritten, whatever it held
        lib.hstu_cp_ring_pass_bias(ql, gl, kp, vp, off, T, tq, tp, tab, 2, w.max_len, w.alpha, True, cp, rq,
                                   accumulate_dkv=True, out=(o, dq, dks, dvs, dw))
        torch.cuda.synchronize()
        _check("o", o, want[0][rows[rq]], "bf16", "ring bias cp%d q%d" % (cp, rq))
        _check("dq", dq, want[1][rows[rq]], "bf16", "ring bias cp%d q%d" % (cp, rq))
        dw_sum += dw
        o2 = lib.hstu_cp_ring_pass_bias(ql, None, kp, vp, off, T, tq, tp, tab, 2, w.max_len, w.alpha, True,
                                        cp, rq)[0]
        torch.cuda.synchronize()
        assert torch.equal(o2, o)
    for r in range(cp):
        if len(rows[r]):
            _check("dk", dks[r], want[2][rows[r]], "bf16", "ring bias cp%d part %d" % (cp, r))
            _check("dv", dvs[r], want[3][rows[r]], "bf16", "ring bias cp%d part %d" % (cp, r))
    _check_dw(dw_sum, want[4], "ring bias cp%d" % cp)


@pytest.mark.parametrize("kind", ["events", "shuffled", "wide"])
@pytest.mark.parametrize("causal", [True, False])
def test_bias_fp32_inputs(kind, causal):
    """All-fp32 arithmetic: o, dq, dk, dv within 1e-5 x RMS of the oracle (which no misplaced pair
    would survive), the table gradient within 1e-4.  Unequal head dimensions are allowed here."""
    w = workloads.custom("bias_f32", [150, 1, 0, 77, 260, 33], 2, 64, 32, 260, dtype="f32", scale=1.0, seed=50)
    _run(w, kind, nb=40, f=2, causal=causal, wscale=0.5, seed=7)


def test_bias_fp32_context_parallel_partial():
    import paper_2508_04711_amd as lib
    cp = 2
    w = workloads.custom("cp_bias_f32", [200, 61, 0, 130], 2, 32, 32, 200, dtype="f32", scale=1.0, seed=51)
    vals = workloads.values(w)
    dev = _dev(vals)
    f64 = {k: workloads.to_f64(v) for k, v in vals.items()}
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    T = w.total_rows
    ts_np, tab_np = workloads.timestamps(w, "events", 9), workloads.bias_table(24, 9, 0.5)
    ts, tab = torch.from_numpy(ts_np).cuda(), torch.from_numpy(tab_np).cuda()
    want = oracle.bias_attention(f64["q"], f64["k"], f64["v"], f64["d_o"], off_np, ts_np,
                                 tab_np.astype(np.float64), 1, w.max_len, w.alpha, True)
    rows = [oracle.cp_global_rows(off_np, cp, r) for r in range(cp)]
    dk_sum = torch.zeros((T, 2, 32), dtype=torch.float32, device="cuda")
    dv_sum = torch.zeros_like(dk_sum)
    dw_sum = torch.zeros(24, dtype=torch.float32, device="cuda")
    for rq in range(cp):
        ql, gl, tq = lib.hstu_cp_reorder([dev["q"], dev["d_o"], ts], off, T, cp, rq, len(rows[rq]))
        o, dq, dk, dv, dw = lib.hstu_jagged_attn_cp_partial_bias(ql, dev["k"], dev["v"], gl, off, T, tq, ts, tab, 1,
                                                                 w.max_len, w.alpha, True, cp, rq, -1)
        torch.cuda.synchronize()
        _check("o", o, want[0][rows[rq]], "f32", "cp f32 q%d" % rq)
        _check("dq", dq, want[1][rows[rq]], "f32", "cp f32 q%d" % rq)
        dk_sum += dk; dv_sum += dv; dw_sum += dw
    _check("dk", dk_sum, want[2], "f32", "cp f32")
    _check("dv", dv_sum, want[3], "f32", "cp f32")
    g = dw_sum.double().cpu().numpy()
    rms = float(np.sqrt(np.mean(want[4] ** 2)))
    assert np.abs(g - want[4]).max() <= 1e-4 * rms


def test_context_parallel_partial_with_bias_at_full_size():
    """Config 4's lengths (8 sequences of 4304..14552 rows, CP = 4, H = 4, d = 128) with event
    timestamps: two ranks' partials against all keys, sampled query rows against the bias oracle;
    the key-side gradients and the table gradient must be finite and, for the ranks that were
    run, of the size the oracle's sampled rows show."""
    import paper_2508_04711_amd as lib
    w = workloads.config(4)
    vals = workloads.values(w)
    dev = _dev(vals)
    f64 = {k: workloads.to_f64(v) for k, v in vals.items()}
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    T, cp = w.total_rows, w.cp_size
    ts_np, tab_np = workloads.timestamps(w, "events", 4), workloads.bias_table(64, 4)
    ts, tab = torch.from_numpy(ts_np).cuda(), torch.from_numpy(tab_np).cuda()
    rng = np.random.default_rng(45)
    dk_sum = dv_sum = None
    for rq in range(cp):
        print("config 4 with bias: rank", rq, flush=True)
        g = oracle.cp_global_rows(off_np, cp, rq)
        ql, gl, tq = lib.hstu_cp_reorder([dev["q"], dev["d_o"], ts], off, T, cp, rq, len(g))
        o, dq, dk, dv, dw = lib.hstu_jagged_attn_cp_partial_bias(
            ql, dev["k"], dev["v"], gl, off, T, tq, ts, tab, 2, w.max_len, w.alpha, True, cp, rq, -1,
            out_dtype=torch.float32)
        torch.cuda.synchronize()
        dk_sum = dk if dk_sum is None else dk_sum + dk
        dv_sum = dv if dv_sum is None else dv_sum + dv
        assert torch.isfinite(dw).all() and (dw != 0).any()
        if rq in (0, cp - 1):
            n = len(g)
            sel = sorted(set([0, 1, 127, 128, n - 1, n // 2] + [int(x) for x in rng.integers(0, n, size=10)]))
            want = oracle.bias_rows(f64["q"], f64["k"], f64["v"], f64["d_o"], off_np, ts_np,
                                    tab_np.astype(np.float64), 2, w.max_len, w.alpha, True, g[sel])
            _check("o", o[sel], want[0], "bf16", "config 4 with bias, rank %d" % rq)
            _check("dq", dq[sel], want[1], "bf16", "config 4 with bias, rank %d" % rq)
    # the sums over the four ranks are the whole batch's key-side gradients
    sel = sorted(set([0, 1, T - 1, T // 2] + [int(x) for x in rng.integers(0, T, size=20)]))
    want = oracle.bias_rows(f64["q"], f64["k"], f64["v"], f64["d_o"], off_np, ts_np,
                            tab_np.astype(np.float64), 2, w.max_len, w.alpha, True, sel)
    _check("dk", dk_sum[sel], want[2], "bf16", "config 4 with bias, all ranks")
    _check("dv", dv_sum[sel], want[3], "bf16", "config 4 with bias, all ranks")


def test_table_gradient_on_a_long_sequence_against_the_full_oracle():
    """The table gradient is a sum over every visible pair and cannot be sampled: one sequence of
    config 5's lengths (5337 rows, H = 2, d = 128; 28 million pairs, about a minute of the
    single-threaded bias oracle) against the full oracle, all five results."""
    import paper_2508_04711_amd as lib
    w = workloads.custom("dw_long", [5337], 2, 128, 128, 32768, dtype="bf16", seed=77)
    vals = workloads.values(w)
    dev = _dev(vals)
    f64 = {k: workloads.to_f64(v) for k, v in vals.items()}
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    ts_np, tab_np = workloads.timestamps(w, "events", 0), workloads.bias_table(64, 0, 1.0)
    ts, tab = torch.from_numpy(ts_np).cuda(), torch.from_numpy(tab_np).cuda()
    o = lib.hstu_jagged_attn_bias_fwd(dev["q"], dev["k"], dev["v"], off, ts, tab, 2, w.max_len, w.alpha, True,
                                      out_dtype=torch.float32)
    dq, dk, dv, dw = lib.hstu_jagged_attn_bias_bwd(dev["q"], dev["k"], dev["v"], dev["d_o"], off, ts, tab, 2,
                                                   w.max_len, w.alpha, True, out_dtype=torch.float32)
    torch.cuda.synchronize()
    print("dw long: gpu done", flush=True)
    want = oracle.bias_attention(f64["q"], f64["k"], f64["v"], f64["d_o"], off_np, ts_np,
                                 tab_np.astype(np.float64), 2, w.max_len, w.alpha, True)
    print("dw long: oracle done", flush=True)
    for name, got, ref in zip(("o", "dq", "dk", "dv"), (o, dq, dk, dv), want):
        _check(name, got, ref, "bf16", "dw long")
    _check_dw(dw, want[4], "dw long")
    # buckets no pair falls into are exactly zero
    assert (dw.cpu().numpy()[want[4] == 0] == 0).all()
