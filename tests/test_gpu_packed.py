"""Packed tiles: batches of very short sequences (bf16; by default a mean length of at most 256,
here forced for every case with HSTU_FLAG_PACK_SHORT) are tiled 128 rows at a time across sequence
boundaries, each row seeing the window of its own sequence.  Against the oracle, through the C
ABI, on the shapes that stress the windows: many sequences per tile, sequences spanning tiles,
empty sequences, one long sequence among short ones, no mask."""
import numpy as np
import pytest
import torch

from conftest import set_flags
import oracle
import workloads
from test_gpu_parity import _check, _check_few_terms, _dev

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _packed(monkeypatch):
    set_flags(monkeypatch, remove="NO_PACK")
    set_flags(monkeypatch, add="PACK_SHORT")


def _run(w, causal=True, out_dtype=torch.float32, few_terms=False):
    import paper_2508_04711_amd as lib
    assert w.total_rows // max(w.batch, 1) <= 1024, "not a packed-tile problem"
    vals = workloads.values(w)
    d = _dev(vals)
    f64 = {k: workloads.to_f64(v) for k, v in vals.items()}
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    tag = "%s/%s" % (w.name, "causal" if causal else "full")
    print("packed", tag, w.total_rows, flush=True)
    o = lib.hstu_jagged_attn_fwd(d["q"], d["k"], d["v"], off, w.max_len, w.alpha, causal, out_dtype=out_dtype)
    dq, dk, dv = lib.hstu_jagged_attn_bwd(d["q"], d["k"], d["v"], d["d_o"], off, w.max_len, w.alpha, causal,
                                          out_dtype=out_dtype)
    torch.cuda.synchronize()
    want_o = oracle.fwd(f64["q"], f64["k"], f64["v"], off_np, w.max_len, w.alpha, causal)
    want = oracle.bwd(f64["q"], f64["k"], f64["v"], f64["d_o"], off_np, w.max_len, w.alpha, causal)
    for name, g, ref in zip(("o", "dq", "dk", "dv"), (o, dq, dk, dv), (want_o,) + tuple(want)):
        if few_terms:
            _check_few_terms(name, g, ref, tag)
        else:
            _check(name, g, ref, w.dtype, tag)
    return o, dq, dk, dv


CASES = [
    ("all_ones", [1] * 300, 2, 64, 64),                                   # 128 sequences per tile
    ("tiny_mix", [3, 1, 0, 7, 2, 0, 0, 5, 1, 9] * 40, 1, 32, 32),
    ("tile_multiples", [128, 256, 128, 384, 128], 2, 128, 128),           # boundaries on tile edges
    ("off_by_one", [127, 129, 1, 255, 257, 63, 65], 2, 64, 64),
    ("one_long_among_short", [20, 2900, 15, 33, 8, 40, 12, 25, 30, 18], 2, 64, 64),  # mean 310
    ("ragged", [200, 1, 0, 77, 300, 5, 0, 131, 510, 64], 3, 128, 64),
    ("dims", [90, 33, 140, 7], 2, 32, 128),
]


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("name,lengths,H,dqk,dv", CASES)
def test_packed_tiles_match_oracle(name, lengths, H, dqk, dv, causal):
    w = workloads.custom(name, lengths, H, dqk, dv, max_len=max(lengths), dtype="bf16", seed=len(lengths) + H)
    _run(w, causal, few_terms=max(lengths) < 16)


def test_packed_bf16_outputs():
    w = workloads.custom("packed_bf16out", [150, 40, 260, 3, 77], 2, 128, 128, 260, dtype="bf16", seed=4)
    _run(w, True, out_dtype=torch.bfloat16)


def test_packed_equals_per_sequence_tiling_closely(monkeypatch):
    """The two tilings add the same terms in another grouping: fp32 outputs agree to rounding."""
    import paper_2508_04711_amd as lib
    rng = np.random.default_rng(5)
    lengths = [int(x) for x in rng.integers(0, 400, size=60)]
    w = workloads.custom("both_tilings", lengths, 2, 64, 64, 400, dtype="bf16", seed=6)
    d = _dev(workloads.values(w))
    off = torch.from_numpy(w.seq_offsets()).cuda()

    def run():
        o = lib.hstu_jagged_attn_fwd(d["q"], d["k"], d["v"], off, w.max_len, w.alpha, True,
                                     out_dtype=torch.float32)
        g = lib.hstu_jagged_attn_bwd(d["q"], d["k"], d["v"], d["d_o"], off, w.max_len, w.alpha, True,
                                     out_dtype=torch.float32)
        torch.cuda.synchronize()
        return (o,) + tuple(g)

    set_flags(monkeypatch, remove="NO_PACK")
    packed = run()
    set_flags(monkeypatch, add="NO_PACK")
    plain = run()
    for name, a, b in zip(("o", "dq", "dk", "dv"), packed, plain):
        scale = b.abs().max().item()
        # P and dS are rounded to bf16 as operands in both; what differs is the order of fp32 sums
        assert (a - b).abs().max().item() <= 1e-4 * scale, name


def test_offsets_that_end_before_the_declared_rows():
    """off[B] < total_rows: the rows beyond belong to no sequence and are not written."""
    import paper_2508_04711_amd as lib
    lengths = [100, 37, 180]
    w = workloads.custom("short_offsets", lengths + [90], 2, 64, 64, 180, dtype="bf16", seed=8)
    d = _dev(workloads.values(w))               # 407 rows of data
    off_np = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)   # ends at 317
    off = torch.from_numpy(off_np).cuda()
    T = w.total_rows
    o = torch.full((T, 2, 64), float("nan"), dtype=torch.float32, device="cuda")
    lib.hstu_jagged_attn_fwd(d["q"], d["k"], d["v"], off, w.max_len, w.alpha, True, out=o)
    torch.cuda.synchronize()
    assert torch.isnan(o[317:]).all() and not torch.isnan(o[:317]).any()
    f64 = {k: workloads.to_f64(v)[:317] for k, v in workloads.values(w).items()}
    want = oracle.fwd(f64["q"], f64["k"], f64["v"], off_np, w.max_len, w.alpha, True)
    _check("o", o[:317], want, "bf16", "short_offsets")


def test_four_thousand_short_sequences():
    """The short-sequence workload at its real batch size (sampled: the oracle on a slice)."""
    import paper_2508_04711_amd as lib
    rng = np.random.default_rng(9)
    lengths = [int(x) for x in rng.integers(32, 257, size=4096)]
    w = workloads.custom("short4096", lengths, 4, 128, 128, 256, dtype="bf16", seed=10)
    vals = workloads.values(w)
    d = _dev(vals)
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).cuda()
    print("short4096", w.total_rows, flush=True)
    o = lib.hstu_jagged_attn_fwd(d["q"], d["k"], d["v"], off, w.max_len, w.alpha, True, out_dtype=torch.float32)
    dq, dk, dv = lib.hstu_jagged_attn_bwd(d["q"], d["k"], d["v"], d["d_o"], off, w.max_len, w.alpha, True,
                                          out_dtype=torch.float32)
    torch.cuda.synchronize()
    # sequences are independent: the oracle on three slices of whole sequences
    for first in (0, 2000, 4076):
        s, e = int(off_np[first]), int(off_np[first + 20])
        sub_off = (off_np[first:first + 21] - s).astype(np.int32)
        f64 = {k: workloads.to_f64(v[s:e]) for k, v in vals.items()}
        want_o = oracle.fwd(f64["q"], f64["k"], f64["v"], sub_off, w.max_len, w.alpha, True)
        want = oracle.bwd(f64["q"], f64["k"], f64["v"], f64["d_o"], sub_off, w.max_len, w.alpha, True)
        _check("o", o[s:e], want_o, "bf16", "short4096@%d" % first)
        for name, g, ref in zip(("dq", "dk", "dv"), (dq, dk, dv), want):
            _check(name, g[s:e], ref, "bf16", "short4096@%d" % first)


# ---- packed tiles with the timestamp bias ---------------------------------------------------

@pytest.mark.parametrize("kind", ["events", "shuffled", "equal", "wide"])
@pytest.mark.parametrize("d", [32, 64, 128])
def test_packed_tiles_with_bias_match_oracle(kind, d):
    """Blocks whose rows belong to several sequences: the ranges a block's one-bucket test uses
    cover the rows of all of them; hidden pairs contribute neither to the outputs nor to dW."""
    from test_gpu_bias import _run as run_bias
    rng = np.random.default_rng(d)
    lengths = [int(x) for x in rng.integers(0, 90, size=40)] + [300, 1, 129, 64]
    w = workloads.custom("packed_bias", lengths, 2, d, d, 300, dtype="bf16", seed=30 + d)
    # (40 of the 44 sequences are shorter than 90 rows: the few-terms bar, see _check_few_terms;
    # measured against the standard bar: 2.03e-2 at d = 128, wide timestamps)
    run_bias(w, kind, nb=40, f=2, causal=True, seed=d, check=_check_few_terms)


def test_packed_tiles_with_bias_no_mask_and_bucket_shapes():
    from test_gpu_bias import _run as run_bias
    lengths = [5, 70, 33, 0, 128, 17, 250, 1, 1, 64] * 4
    w = workloads.custom("packed_bias_full", lengths, 3, 64, 64, 250, dtype="bf16", seed=7)
    run_bias(w, "events", nb=24, f=1, causal=False, seed=1)
    run_bias(w, "events", nb=1, f=0, causal=True, seed=2)
    run_bias(w, "wide", nb=512, f=4, causal=True, out_dtype=torch.bfloat16, seed=3)


def test_packed_bias_table_gradient_equals_per_sequence_tiles(monkeypatch):
    """The same call with packed and with per-sequence tiles, 36 K rows in 600 sequences: the
    outputs agree to operand rounding and the table gradient, a sum over the same visible pairs,
    to fp32 summation error."""
    import paper_2508_04711_amd as lib
    rng = np.random.default_rng(3)
    lengths = [int(x) for x in rng.integers(1, 120, size=600)]
    w = workloads.custom("packed_bias_many", lengths, 4, 128, 128, 120, dtype="bf16", seed=12)
    dev = _dev(workloads.values(w))
    off = torch.from_numpy(w.seq_offsets()).cuda()
    ts = torch.from_numpy(workloads.timestamps(w, "events", 4)).cuda()
    tab = torch.from_numpy(workloads.bias_table(64, 4)).cuda()
    def run(packed, per_pair):
        set_flags(monkeypatch, remove="NO_PACK" if packed else "", add="" if packed else "NO_PACK")
        set_flags(monkeypatch, add="BIAS_PER_PAIR" if per_pair else "", remove="" if per_pair else "BIAS_PER_PAIR")
        o = lib.hstu_jagged_attn_bias_fwd(dev["q"], dev["k"], dev["v"], off, ts, tab, 2, w.max_len, w.alpha, True,
                                          out_dtype=torch.float32)
        g = lib.hstu_jagged_attn_bias_bwd(dev["q"], dev["k"], dev["v"], dev["d_o"], off, ts, tab, 2, w.max_len,
                                          w.alpha, True, out_dtype=torch.float32)
        torch.cuda.synchronize()
        return (o,) + tuple(g)
    # As the calls run by default, the two forms see a block's table entry as hi + lo bf16 halves or
    # as the fp32 value depending on which blocks each of them finds to be of one bucket, so scores
    # differ in the 16th bit and a P or dS operand may round to the other bf16 neighbour: one term
    # of a handful moves by 2^-8 of its value.  The table gradient sums fp32 dS values that are
    # never rounded.
    a4, b4 = run(True, False), run(False, False)
    for name, a, b in zip(("o", "dq", "dk", "dv", "dw"), a4, b4):
        a, b = a.double(), b.double()
        rms = float(b.pow(2).mean().sqrt())
        print("packed vs tiled", name, float((a - b).abs().max()) / rms, flush=True)
        if name == "dw":
            assert float((a - b).abs().max()) <= 2e-3 * rms
        else:
            assert bool(((a - b).abs() <= 1e-2 * rms + b.abs() * 2.0 ** -7).all()), name
    # That this is the whole difference: with every block on the per-pair path both forms see the
    # same fp32 entries, hence the same scores and the same bf16 operands, and what remains is the
    # order of fp32 additions.
    a4, b4 = run(True, True), run(False, True)
    for name, a, b in zip(("o", "dq", "dk", "dv", "dw"), a4, b4):
        a, b = a.double(), b.double()
        rms = float(b.pow(2).mean().sqrt())
        print("packed vs tiled, per-pair entries", name, float((a - b).abs().max()) / rms, flush=True)
        assert float((a - b).abs().max()) <= (1e-4 if name == "dw" else 1e-5) * rms, name
