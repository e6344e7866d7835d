"""Context-parallel partials on the GPU against the oracle and against the GPU's own full pass."""
import numpy as np
import pytest
import torch

from conftest import set_flags
import oracle
import workloads
from test_gpu_parity import _check, _dev

pytestmark = pytest.mark.gpu


def _gather(vals, idx):
    return {k: v[idx].contiguous() for k, v in vals.items()}


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("cp", [1, 2, 4])
def test_rank_pairs_match_oracle_and_add_up(cp, dtype):
    import paper_2508_04711_amd as lib
    lengths = [160, 5, 233, 1, 0, 384, 77]
    w = workloads.custom("cp_small", lengths, 2, 64, 64, 384, dtype=dtype,
                         scale=1.0 if dtype == "f32" else 0.5, seed=cp)
    vals = workloads.values(w)
    dev = _dev(vals)
    f64 = {k: workloads.to_f64(v) for k, v in vals.items()}
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    T = w.total_rows
    rows = [oracle.cp_global_rows(off_np, cp, r) for r in range(cp)]
    trow = [torch.from_numpy(r).cuda() for r in rows]
    want_o = oracle.fwd(f64["q"], f64["k"], f64["v"], off_np, w.max_len, w.alpha, True)
    want_g = oracle.bwd(f64["q"], f64["k"], f64["v"], f64["d_o"], off_np, w.max_len, w.alpha, True)
    dk_sum = torch.zeros((T, 2, 64), dtype=torch.float32, device="cuda")
    dv_sum = torch.zeros((T, 2, 64), dtype=torch.float32, device="cuda")
    for rq in range(cp):
        ql = _gather(dev, trow[rq])
        # one key rank at a time, accumulated in fp32 as ring steps would be
        o_acc = torch.zeros((len(rows[rq]), 2, 64), dtype=torch.float32, device="cuda")
        dq_acc = torch.zeros_like(o_acc)
        for rk in range(cp):
            kl = _gather(dev, trow[rk])
            print("pair", cp, rq, rk, dtype, flush=True)
            # stand-alone partial against the oracle's partial
            o, dq, dk, dv = lib.hstu_jagged_attn_cp_partial(
                ql["q"], kl["k"], kl["v"], ql["d_o"], off, T, w.max_len, w.alpha, True, cp, rq, rk,
                out_dtype=torch.float32)
            wo, wdq, wdk, wdv = oracle.cp_partial(
                f64["q"][rows[rq]], f64["k"][rows[rk]], f64["v"][rows[rk]], f64["d_o"][rows[rq]],
                off_np, w.max_len, w.alpha, True, cp, rq, rk)
            tag = "cp%d q%d kv%d" % (cp, rq, rk)
            # a pair with nothing visible is exactly zero on both sides
            for name, g, ref in (("o", o, wo), ("dq", dq, wdq), ("dk", dk, wdk), ("dv", dv, wdv)):
                if not np.any(ref):
                    assert not torch.any(g), tag + " " + name
                else:
                    _check(name, g, ref, dtype, tag)
            # the same step with accumulate = 1 into running fp32 sums
            dk_run = torch.zeros((len(rows[rk]), 2, 64), dtype=torch.float32, device="cuda")
            dv_run = torch.zeros_like(dk_run)
            lib.hstu_jagged_attn_cp_partial(
                ql["q"], kl["k"], kl["v"], ql["d_o"], off, T, w.max_len, w.alpha, True, cp, rq, rk,
                accumulate=True, out=(o_acc, dq_acc, dk_run, dv_run))
            dk_sum[trow[rk]] += dk_run
            dv_sum[trow[rk]] += dv_run
        _check("o sum", o_acc, want_o[rows[rq]], dtype, "cp%d q%d" % (cp, rq))
        _check("dq sum", dq_acc, want_g[0][rows[rq]], dtype, "cp%d q%d" % (cp, rq))
    _check("dk sum", dk_sum, want_g[1], dtype, "cp%d" % cp)
    _check("dv sum", dv_sum, want_g[2], dtype, "cp%d" % cp)


def test_all_keys_partial_is_bitwise_the_full_pass(monkeypatch):
    # kv_rank = -1 streams the same key tiles in the same order as whole-batch attention, and a
    # query row's result does not depend on which other rows share its tile.  (With the cutting
    # of heavy query tiles along the keys switched off: how many parts a tile is cut into depends
    # on the number of query rows of the call, and the parts are summed in another order; and with
    # the whole-batch call tiled per sequence like the partial, not with packed tiles.)
    import paper_2508_04711_amd as lib
    set_flags(monkeypatch, add="NO_SPLIT")
    set_flags(monkeypatch, add="NO_PACK")
    lengths = [520, 96, 1030, 8]
    w = workloads.custom("cp_all", lengths, 2, 128, 128, 1030, dtype="bf16", seed=9)
    dev = _dev(workloads.values(w))
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    T, cp = w.total_rows, 4
    o_full = lib.hstu_jagged_attn_fwd(dev["q"], dev["k"], dev["v"], off, w.max_len, w.alpha, True)
    dq_full, dk_full, dv_full = lib.hstu_jagged_attn_bwd(dev["q"], dev["k"], dev["v"], dev["d_o"], off,
                                                         w.max_len, w.alpha, True, out_dtype=torch.float32)
    dk_sum = torch.zeros_like(dk_full); dv_sum = torch.zeros_like(dv_full)
    for r in range(cp):
        idx = torch.from_numpy(oracle.cp_global_rows(off_np, cp, r)).cuda()
        ql = _gather(dev, idx)
        o, _, _, _ = lib.hstu_jagged_attn_cp_partial(ql["q"], dev["k"], dev["v"], None, off, T,
                                                    w.max_len, w.alpha, True, cp, r, -1)
        assert torch.equal(o, o_full[idx])
        _, dq, dk, dv = lib.hstu_jagged_attn_cp_partial(ql["q"], dev["k"], dev["v"], ql["d_o"], off, T,
                                                       w.max_len, w.alpha, True, cp, r, -1,
                                                       want_o=False, out_dtype=torch.float32)
        assert torch.equal(dq, dq_full[idx])
        dk_sum += dk; dv_sum += dv
    # key-side sums over ranks run in another order than the full pass: equal to rounding
    scale = dk_full.abs().max().item()
    assert (dk_sum - dk_full).abs().max().item() <= 1e-4 * scale
    assert (dv_sum - dv_full).abs().max().item() <= 1e-4 * dv_full.abs().max().item()


def test_config4_every_rank_sampled():
    """Config 4 at full size: each of the 4 ranks against all visible keys, sampled rows exact."""
    import paper_2508_04711_amd as lib
    w = workloads.config(4)
    vals = workloads.values(w)
    dev = _dev(vals)
    f64 = {k: workloads.to_f64(v) for k, v in vals.items()}
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    T, cp = w.total_rows, w.cp_size
    rng = np.random.default_rng(4)
    dk_sum = torch.zeros((T, w.num_heads, w.d_qk), dtype=torch.float32, device="cuda")
    dv_sum = torch.zeros((T, w.num_heads, w.d_v), dtype=torch.float32, device="cuda")
    for r in range(cp):
        print("config 4 rank", r, flush=True)
        g = oracle.cp_global_rows(off_np, cp, r)
        assert len(g) == T // cp                     # lengths are multiples of 2*CP: equal shares
        idx = torch.from_numpy(g).cuda()
        ql = _gather(dev, idx)
        o, dq, dk, dv = lib.hstu_jagged_attn_cp_partial(ql["q"], dev["k"], dev["v"], ql["d_o"], off, T,
                                                       w.max_len, w.alpha, True, cp, r, -1,
                                                       out_dtype=torch.float32)
        torch.cuda.synchronize()
        dk_sum += dk; dv_sum += dv
        # exact oracle values at sampled local query rows: chunk edges, tile edges, random
        nloc = len(g)
        edges = [0, 1, 127, 128, 129, nloc - 1, nloc - 2, nloc // 2]
        sel = sorted(set(edges + [int(x) for x in rng.integers(0, nloc, size=24)]))
        so, sdq, sdk, sdv = oracle.rows(f64["q"], f64["k"], f64["v"], f64["d_o"], off_np, w.max_len,
                                        w.alpha, True, g[sel])
        rms_o = float(np.sqrt((so ** 2).mean())); rms_q = float(np.sqrt((sdq ** 2).mean()))
        eo = np.abs(o[sel].double().cpu().numpy() - so).max() / rms_o
        eq = np.abs(dq[sel].double().cpu().numpy() - sdq).max() / rms_q
        assert eo <= 2e-2 and eq <= 2e-2, (r, eo, eq)
    # sum over ranks of the key-side partials = full dK, dV (sampled global rows)
    sel = sorted(set([0, 1, T - 1, T // 2] + [int(x) for x in rng.integers(0, T, size=40)]))
    _, _, sdk, sdv = oracle.rows(f64["q"], f64["k"], f64["v"], f64["d_o"], off_np, w.max_len, w.alpha,
                                 True, sel)
    ek = np.abs(dk_sum[sel].double().cpu().numpy() - sdk).max() / float(np.sqrt((sdk ** 2).mean()))
    ev = np.abs(dv_sum[sel].double().cpu().numpy() - sdv).max() / float(np.sqrt((sdv ** 2).mean()))
    assert ek <= 2e-2 and ev <= 2e-2, (ek, ev)


@pytest.mark.parametrize("cp", [2, 4])
def test_large_batch_rank_partials_against_all_keys(cp):
    """4096 sequences of 64..512 rows, H = 4, d = 128: a batch large enough for the natural item
    order, the XCD-aware workgroup map and the dK/dV workgroups that walk over items, here with the
    two-segment items of a context-parallel rank.  Every rank's partial against all keys (as the
    benchmark runs them), scattered back; sampled sequences against the oracle's full attention."""
    import paper_2508_04711_amd as lib
    rng = np.random.default_rng(31 + cp)
    B, H, d = 4096, 4, 128
    lengths = [int(x) for x in rng.integers(64, 513, size=B)]
    w = workloads.custom("cp_large_batch", lengths, H, d, d, 512, dtype="bf16", seed=60 + cp)
    dev = workloads.device_values(w)
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    T = w.total_rows
    # fp32 outputs: the sums of the ranks' partial results then carry no rounding between ranks, and
    # the stated bar applies as it is
    o = torch.zeros((T, H, d), dtype=torch.float32, device="cuda")
    dq = torch.zeros_like(o)
    dk = torch.zeros_like(o)
    dv = torch.zeros_like(o)
    for r in range(cp):
        n = len(oracle.cp_global_rows(off_np, cp, r))
        print("cp large batch", cp, r, n, flush=True)
        ql, gl = lib.hstu_cp_reorder([dev["q"], dev["d_o"]], off, T, cp, r, n)
        ol, dql, dkp, dvp = lib.hstu_jagged_attn_cp_partial(ql, dev["k"], dev["v"], gl, off, T, w.max_len, w.alpha,
                                                            True, cp, r, -1, out_dtype=torch.float32)
        lib.hstu_cp_reorder([ol, dql], off, T, cp, r, n, scatter=True, out=[o, dq])
        dk += dkp
        dv += dvp
    torch.cuda.synchronize()
    seqs = [0, 1, B // 2 - 1, B // 2, B - 2, B - 1]
    rows = np.concatenate([np.arange(off_np[b], off_np[b + 1]) for b in seqs])
    rows_t = torch.from_numpy(rows).cuda()
    sub = {k: workloads.to_f64(v[rows_t]) for k, v in dev.items()}
    sub_off = np.concatenate([[0], np.cumsum([lengths[b] for b in seqs])]).astype(np.int32)
    want = oracle.rows(sub["q"], sub["k"], sub["v"], sub["d_o"], sub_off, w.max_len, w.alpha, True,
                       np.arange(len(rows)))
    for name, got, ref in zip(("o", "dq", "dk", "dv"), (o, dq, dk, dv), want):
        _check(name, got[rows_t], ref, "bf16", "cp large batch, cp=%d" % cp)
    for t in (o, dq, dk, dv):
        assert torch.isfinite(t).all()
