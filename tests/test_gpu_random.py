"""Seeded random problems against the oracle: mixed lengths (empty, shorter than a tile, several
tiles, long enough for tiles to be cut along the keys), head counts, head dimensions, causal or
not, whole-batch and context-parallel.  Each case is small enough for the full oracle."""
import numpy as np
import pytest
import torch

from conftest import set_flags
import oracle
import workloads
from test_gpu_parity import _check, _dev

pytestmark = pytest.mark.gpu


def _case(seed):
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.integers(1, 6))
    pools = [lambda: 0, lambda: int(rng.integers(1, 40)), lambda: int(rng.integers(40, 700)),
             lambda: int(rng.integers(700, 1800)), lambda: int(rng.integers(4096, 5200))]
    weights = [0.1, 0.25, 0.35, 0.2, 0.1]
    lengths = [pools[int(rng.choice(5, p=weights))]() for _ in range(n)]
    if seed % 3 == 0:
        lengths[int(rng.integers(0, n))] = int(rng.integers(4096, 5200))   # make the cutting likely
    H = int(rng.choice([1, 2, 3]))
    dqk, dv = [(32, 32), (64, 64), (128, 128), (128, 64), (64, 128), (32, 128)][int(rng.integers(0, 6))]
    causal = bool(rng.integers(0, 4) > 0)
    cp = [0, 0, 2, 3][int(rng.integers(0, 4))]
    return lengths, H, dqk, dv, causal, cp


@pytest.mark.parametrize("tiling", ["default", "packed"])
@pytest.mark.parametrize("seed", range(14))
def test_random_problem(seed, tiling, monkeypatch):
    import paper_2508_04711_amd as lib
    lengths, H, dqk, dv, causal, cp = _case(seed)
    set_flags(monkeypatch, remove="NO_PACK")
    if tiling == "packed":   # packed tiles forced for every batch they can serve
        if cp or sum(lengths) // len(lengths) > 1024:
            pytest.skip("tiled per sequence whatever the threshold")
        set_flags(monkeypatch, add="PACK_SHORT")
    if sum(lengths) == 0:
        lengths = lengths + [17]
    w = workloads.custom("rand%d" % seed, lengths, H, dqk, dv, max_len=max(max(lengths), 1), dtype="bf16",
                         seed=seed)
    print("random", seed, lengths, H, dqk, dv, causal, cp, flush=True)
    vals = workloads.values(w)
    d = _dev(vals)
    f64 = {k: workloads.to_f64(v) for k, v in vals.items()}
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    T = w.total_rows
    want_o = oracle.fwd(f64["q"], f64["k"], f64["v"], off_np, w.max_len, w.alpha, causal)
    wq, wk, wv = oracle.bwd(f64["q"], f64["k"], f64["v"], f64["d_o"], off_np, w.max_len, w.alpha, causal)
    tag = "rand%d" % seed
    if cp == 0:
        o = lib.hstu_jagged_attn_fwd(d["q"], d["k"], d["v"], off, w.max_len, w.alpha, causal,
                                     out_dtype=torch.float32)
        dq, dk, dvv = lib.hstu_jagged_attn_bwd(d["q"], d["k"], d["v"], d["d_o"], off, w.max_len, w.alpha,
                                               causal, out_dtype=torch.float32)
        for name, g, ref in (("o", o, want_o), ("dq", dq, wq), ("dk", dk, wk), ("dv", dvv, wv)):
            _check(name, g, ref, "bf16", tag)
        return
    # context-parallel: every rank against all keys (reorder in, partial, reorder out), sums over ranks
    o_glob = torch.zeros((T, H, dv), dtype=torch.float32, device="cuda")
    dq_glob = torch.zeros((T, H, dqk), dtype=torch.float32, device="cuda")
    dk_sum = torch.zeros((T, H, dqk), dtype=torch.float32, device="cuda")
    dv_sum = torch.zeros((T, H, dv), dtype=torch.float32, device="cuda")
    for r in range(cp):
        rows = oracle.cp_global_rows(off_np, cp, r)
        ql, gl = lib.hstu_cp_reorder([d["q"], d["d_o"]], off, T, cp, r, len(rows))
        o, dq, dk, dvv = lib.hstu_jagged_attn_cp_partial(ql, d["k"], d["v"], gl, off, T, w.max_len, w.alpha,
                                                        causal, cp, r, -1, out_dtype=torch.float32)
        lib.hstu_cp_reorder([o, dq], off, T, cp, r, len(rows), scatter=True, out=[o_glob, dq_glob])
        dk_sum += dk
        dv_sum += dvv
    for name, g, ref in (("o", o_glob, want_o), ("dq", dq_glob, wq), ("dk", dk_sum, wk), ("dv", dv_sum, wv)):
        _check(name, g, ref, "bf16", tag + " cp%d" % cp)
