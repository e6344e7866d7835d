"""The ring pass of one context-parallel rank (K/V parts arriving step by step, transfers on a
second stream) against the oracle and against the same rank's single launch over all keys."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from test_gpu_parity import _check, _dev

pytestmark = pytest.mark.gpu


def _parts(dev, rows):
    return [dev["k"][r].contiguous() for r in rows], [dev["v"][r].contiguous() for r in rows]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("cp", [1, 2, 3, 4])
def test_ring_matches_oracle_and_sums_to_full_gradients(cp, dtype):
    import paper_2508_04711_amd as lib
    lengths = [160, 5, 233, 1, 0, 384, 77]
    w = workloads.custom("ring_small", lengths, 2, 64, 64, 384, dtype=dtype,
                         scale=1.0 if dtype == "f32" else 0.5, seed=10 + cp)
    vals = workloads.values(w)
    dev = _dev(vals)
    f64 = {k: workloads.to_f64(v) for k, v in vals.items()}
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    T = w.total_rows
    rows = [oracle.cp_global_rows(off_np, cp, r) for r in range(cp)]
    trow = [torch.from_numpy(r).cuda() for r in rows]
    kp, vp = _parts(dev, trow)
    want_o = oracle.fwd(f64["q"], f64["k"], f64["v"], off_np, w.max_len, w.alpha, True)
    want_dq, want_dk, want_dv = oracle.bwd(f64["q"], f64["k"], f64["v"], f64["d_o"], off_np, w.max_len,
                                           w.alpha, True)
    # the key-side gradient buffers travel with their parts: every rank adds its contribution
    dks = [torch.zeros((len(rows[r]), 2, 64), dtype=torch.float32, device="cuda") for r in range(cp)]
    dvs = [torch.zeros((len(rows[r]), 2, 64), dtype=torch.float32, device="cuda") for r in range(cp)]
    for rq in range(cp):
        print("ring", cp, rq, dtype, flush=True)
        ql, gl = dev["q"][trow[rq]].contiguous(), dev["d_o"][trow[rq]].contiguous()
        nq = len(rows[rq])
        o = torch.empty((nq, 2, 64), dtype=torch.float32, device="cuda")
        dq = torch.empty((nq, 2, 64), dtype=torch.float32, device="cuda")
        lib.hstu_cp_ring_pass(ql, gl, kp, vp, off, T, w.max_len, w.alpha, True, cp, rq,
                              accumulate_dkv=True, out=(o, dq, dks, dvs))
        torch.cuda.synchronize()
        _check("o", o, want_o[rows[rq]], dtype, "ring cp%d q%d" % (cp, rq))
        _check("dq", dq, want_dq[rows[rq]], dtype, "ring cp%d q%d" % (cp, rq))
        # forward only gives the same o
        o2, none_dq, none_dk, none_dv = lib.hstu_cp_ring_pass(ql, None, kp, vp, off, T, w.max_len, w.alpha,
                                                               True, cp, rq)
        torch.cuda.synchronize()
        assert none_dq is None and none_dk is None and none_dv is None
        assert torch.equal(o2, o)
    for r in range(cp):
        if len(rows[r]):
            _check("dk", dks[r], want_dk[rows[r]], dtype, "ring cp%d part %d" % (cp, r))
            _check("dv", dvs[r], want_dv[rows[r]], dtype, "ring cp%d part %d" % (cp, r))


def test_ring_equals_step_by_step_partials_bitwise():
    """The ring is the sequence of partials kv_rank = q, q-1, ... with fp32 accumulation: the
    same calls made one by one on one stream give the same bits."""
    import paper_2508_04711_amd as lib
    lengths = [700, 130, 1, 519]
    w = workloads.custom("ring_bits", lengths, 2, 128, 128, 700, dtype="bf16", seed=3)
    dev = _dev(workloads.values(w))
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    T, cp = w.total_rows, 4
    trow = [torch.from_numpy(oracle.cp_global_rows(off_np, cp, r)).cuda() for r in range(cp)]
    kp, vp = _parts(dev, trow)
    for rq in (0, 3):
        ql, gl = dev["q"][trow[rq]].contiguous(), dev["d_o"][trow[rq]].contiguous()
        o, dq, dks, dvs = lib.hstu_cp_ring_pass(ql, gl, kp, vp, off, T, w.max_len, w.alpha, True, cp, rq)
        torch.cuda.synchronize()
        o_ref = torch.zeros_like(o); dq_ref = torch.zeros_like(dq)
        for s in range(cp):
            rk = (rq - s) % cp
            dk_ref = torch.zeros_like(dks[rk]); dv_ref = torch.zeros_like(dvs[rk])
            # accumulate into cleared buffers: the same additions as overwrite-then-accumulate
            lib.hstu_jagged_attn_cp_partial(ql, kp[rk], vp[rk], gl, off, T, w.max_len, w.alpha, True, cp,
                                            rq, rk, accumulate=(s > 0), out=(o_ref, dq_ref, dk_ref, dv_ref))
            assert torch.equal(dk_ref, dks[rk]) and torch.equal(dv_ref, dvs[rk])
        assert torch.equal(o_ref, o) and torch.equal(dq_ref, dq)


def test_ring_on_the_context_parallel_workload_at_full_size():
    """Config 4 at full size (8 sequences of 4304..14552 rows, CP = 4): every rank's ring pass over
    the four parts.  Sampled rows of o and dq of every rank, and of the key-side gradients that
    travelled with the parts through all four ranks, against the oracle (exact rows: rows do not
    interact); two ranks also against their one launch over all keys (the same terms in another
    order)."""
    import paper_2508_04711_amd as lib
    w = workloads.config(4)
    vals = workloads.values(w)
    dev = _dev(vals)
    f64 = {k: workloads.to_f64(v) for k, v in vals.items()}
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    T, cp, H = w.total_rows, w.cp_size, w.num_heads
    rows = [oracle.cp_global_rows(off_np, cp, r) for r in range(cp)]
    trow = [torch.from_numpy(r).cuda() for r in rows]
    kp, vp = _parts(dev, trow)
    dks = [torch.zeros((len(rows[r]), H, w.d_qk), dtype=torch.float32, device="cuda") for r in range(cp)]
    dvs = [torch.zeros((len(rows[r]), H, w.d_v), dtype=torch.float32, device="cuda") for r in range(cp)]
    rng = np.random.default_rng(44)
    for rq in range(cp):
        print("ring config 4 rank", rq, flush=True)
        ql, gl = dev["q"][trow[rq]].contiguous(), dev["d_o"][trow[rq]].contiguous()
        nq = len(rows[rq])
        o = torch.empty((nq, H, w.d_v), dtype=torch.float32, device="cuda")
        dq = torch.empty((nq, H, w.d_qk), dtype=torch.float32, device="cuda")
        lib.hstu_cp_ring_pass(ql, gl, kp, vp, off, T, w.max_len, w.alpha, True, cp, rq,
                              accumulate_dkv=True, out=(o, dq, dks, dvs))
        torch.cuda.synchronize()
        # local rows: the ends of the two mini-chunks of the first and last sequences, tile edges, random
        sel = sorted(set([0, 1, 127, 128, nq - 1, nq - 2, nq // 2] + [int(x) for x in rng.integers(0, nq, size=16)]))
        so, sdq, _, _ = oracle.rows(f64["q"], f64["k"], f64["v"], f64["d_o"], off_np, w.max_len, w.alpha, True,
                                    rows[rq][sel])
        _check("o", o[sel], so, "bf16", "ring config 4 rank %d" % rq)
        _check("dq", dq[sel], sdq, "bf16", "ring config 4 rank %d" % rq)
        if rq in (0, cp - 1):
            o1, dq1, _, _ = lib.hstu_jagged_attn_cp_partial(ql, dev["k"], dev["v"], gl, off, T, w.max_len, w.alpha,
                                                            True, cp, rq, -1, out_dtype=torch.float32)
            torch.cuda.synchronize()
            for name, a, b in (("o", o, o1), ("dq", dq, dq1)):
                assert (a - b).abs().max().item() <= 1e-4 * b.abs().max().item(), name
    # the key-side gradients have now collected every rank's contribution
    for r in range(cp):
        n = len(rows[r])
        sel = sorted(set([0, 1, n - 1, n // 2] + [int(x) for x in rng.integers(0, n, size=12)]))
        _, _, sdk, sdv = oracle.rows(f64["q"], f64["k"], f64["v"], f64["d_o"], off_np, w.max_len, w.alpha, True,
                                     rows[r][sel])
        _check("dk", dks[r][sel], sdk, "bf16", "ring config 4 part %d" % r)
        _check("dv", dvs[r][sel], sdv, "bf16", "ring config 4 part %d" % r)


def test_ring_argument_errors():
    import paper_2508_04711_amd as lib
    w = workloads.custom("ring_err", [64, 64], 1, 32, 32, 64, dtype="bf16", seed=1)
    dev = _dev(workloads.values(w))
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    trow = [torch.from_numpy(oracle.cp_global_rows(off_np, 2, r)).cuda() for r in range(2)]
    kp, vp = _parts(dev, trow)
    ql = dev["q"][trow[0]].contiguous()
    s = torch.cuda.current_stream()
    with pytest.raises(lib.HstuError) as e:      # the two streams must differ
        lib.hstu_cp_ring_pass(ql, None, kp, vp, off, w.total_rows, 64, w.alpha, True, 2, 0, stream=s,
                              copy_stream=s)
    assert e.value.status == -3
    with pytest.raises(lib.HstuError) as e:      # rank out of range
        lib.hstu_cp_ring_pass(ql, None, kp, vp, off, w.total_rows, 64, w.alpha, True, 2, 2)
    assert e.value.status == -5
    small = [torch.empty((8, 1, 32), dtype=torch.bfloat16, device="cuda") for _ in range(4)]
    with pytest.raises(lib.HstuError) as e:      # receive buffers smaller than a part
        lib.hstu_cp_ring_pass(ql, None, kp, vp, off, w.total_rows, 64, w.alpha, True, 2, 0, recv=small)
    assert e.value.status == -5
    with pytest.raises(ValueError):
        lib.hstu_cp_ring_pass(ql, None, kp[:1], vp[:1], off, w.total_rows, 64, w.alpha, True, 2, 0)
