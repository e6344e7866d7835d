"""The library under HIP graph capture: every call is a fixed sequence of kernel launches on the
caller's stream (no allocation, no memset, no host synchronisation, the schedule is built on the
device), so a forward + backward step can be captured once and replayed.  Each replay is checked
against the eager result for the data then in the input buffers."""
import pytest
import torch

from conftest import set_flags
import workloads

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("lengths,H,d", [([700, 130, 1, 519, 0, 64], 2, 128), ([4700, 300], 1, 64)])
def test_forward_backward_step_replays_from_a_graph(lengths, H, d):
    import paper_2508_04711_amd as lib
    w = workloads.custom("graph", lengths, H, d, d, max_len=max(lengths), dtype="bf16", seed=12)
    vals = {k: v.cuda() for k, v in workloads.values(w).items()}
    off = torch.from_numpy(w.seq_offsets()).cuda()
    T = w.total_rows
    p = (w.batch, H, d, d, w.max_len, w.alpha, True, 0, T)
    ws = torch.empty(max(lib.hstu_jagged_attn_workspace_bytes(p, 0), lib.hstu_jagged_attn_workspace_bytes(p, 1)),
                     dtype=torch.uint8, device="cuda")
    # static buffers the graph reads and writes
    q, k, v, g = (vals[n].clone() for n in ("q", "k", "v", "d_o"))
    o = torch.empty((T, H, d), dtype=torch.bfloat16, device="cuda")
    dq, dk, dv = torch.empty_like(o), torch.empty_like(o), torch.empty_like(o)

    def step():
        lib.hstu_jagged_attn_fwd(q, k, v, off, w.max_len, w.alpha, True, out=o, workspace=ws)
        lib.hstu_jagged_attn_bwd(q, k, v, g, off, w.max_len, w.alpha, True, out=(dq, dk, dv), workspace=ws)

    step()                                   # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    gen = torch.Generator(device="cpu").manual_seed(99)
    for it in range(4):
        print("graph replay", it, flush=True)
        # new data in the same buffers, with eager work and a synchronisation between replays
        for t in (q, k, v, g):
            t.copy_((torch.randn(t.shape, generator=gen) * 0.5).to(torch.bfloat16).cuda())
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [x.clone() for x in (o, dq, dk, dv)]
        o.zero_(); dq.zero_(); dk.zero_(); dv.zero_()
        step()                               # eager, same buffers
        torch.cuda.synchronize()
        for name, a, b in zip(("o", "dq", "dk", "dv"), got, (o, dq, dk, dv)):
            assert torch.equal(a, b), (name, it)
            assert torch.isfinite(a.float()).all()


def test_step_with_timestamp_bias_replays_from_a_graph():
    """The calls with bias add one small kernel (the per-row records; it also clears the table
    gradient, so no memset is recorded) and fp32 atomics for the table gradient: dq, dk, dv and o
    replay bit for bit, the table gradient to the rounding of its atomics."""
    import paper_2508_04711_amd as lib
    lengths, H, d = [700, 130, 1, 519, 0, 64], 2, 64
    w = workloads.custom("graph_bias", lengths, H, d, d, max_len=max(lengths), dtype="bf16", seed=13)
    vals = {k: v.cuda() for k, v in workloads.values(w).items()}
    off = torch.from_numpy(w.seq_offsets()).cuda()
    ts = torch.from_numpy(workloads.timestamps(w, "events", 2)).cuda()
    tab = torch.from_numpy(workloads.bias_table(40, 2)).cuda()
    T = w.total_rows
    p = (w.batch, H, d, d, w.max_len, w.alpha, True, 0, T)
    ws = torch.empty(max(lib.hstu_jagged_attn_bias_workspace_bytes(p, 0),
                         lib.hstu_jagged_attn_bias_workspace_bytes(p, 1)), dtype=torch.uint8, device="cuda")
    q, k, v, g = (vals[n].clone() for n in ("q", "k", "v", "d_o"))
    o = torch.empty((T, H, d), dtype=torch.bfloat16, device="cuda")
    dq, dk, dv = torch.empty_like(o), torch.empty_like(o), torch.empty_like(o)
    dw = torch.empty_like(tab)

    def step():
        lib.hstu_jagged_attn_bias_fwd(q, k, v, off, ts, tab, 2, w.max_len, w.alpha, True, out=o, workspace=ws)
        lib.hstu_jagged_attn_bias_bwd(q, k, v, g, off, ts, tab, 2, w.max_len, w.alpha, True,
                                      out=(dq, dk, dv, dw), workspace=ws)

    step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    gen = torch.Generator(device="cpu").manual_seed(7)
    for it in range(3):
        print("graph replay with bias", it, flush=True)
        for t in (q, k, v, g):
            t.copy_((torch.randn(t.shape, generator=gen) * 0.5).to(torch.bfloat16).cuda())
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [x.clone() for x in (o, dq, dk, dv, dw)]
        for t in (o, dq, dk, dv, dw):
            t.zero_()
        step()
        torch.cuda.synchronize()
        for name, a, b in zip(("o", "dq", "dk", "dv"), got, (o, dq, dk, dv)):
            assert torch.equal(a, b), (name, it)
        scale = dw.abs().max().item()
        assert (got[4] - dw).abs().max().item() <= 1e-5 * scale


@pytest.mark.parametrize("mode", ["per_sequence", "packed"])
def test_large_batch_step_replays_from_a_graph(mode, monkeypatch):
    """A batch large enough for the natural item order, the map that gives every XCD one head and
    the dK/dV workgroups that walk over items (per-sequence tiles), and the same batch with
    packed tiles: these paths read the item count on the device and launch fixed grids, so they
    capture and replay like the others."""
    import numpy as np
    import paper_2508_04711_amd as lib
    if mode == "packed":
        set_flags(monkeypatch, add="PACK_SHORT")
    else:
        set_flags(monkeypatch, add="NO_PACK")
    rng = np.random.default_rng(31)
    lengths = [int(x) for x in rng.integers(32, 257, size=4096)]
    H, d = 4, 128
    w = workloads.custom("graph_large", lengths, H, d, d, max_len=256, dtype="bf16", seed=14)
    off = torch.from_numpy(w.seq_offsets()).cuda()
    T = w.total_rows
    p = (w.batch, H, d, d, w.max_len, w.alpha, True, 0, T)
    ws = torch.empty(max(lib.hstu_jagged_attn_workspace_bytes(p, 0), lib.hstu_jagged_attn_workspace_bytes(p, 1)),
                     dtype=torch.uint8, device="cuda")
    gen = torch.Generator(device="cuda").manual_seed(5)

    def fresh():
        return (torch.randn((T, H, d), generator=gen, device="cuda") * 0.5).to(torch.bfloat16)

    q, k, v, g = fresh(), fresh(), fresh(), fresh()
    o = torch.empty((T, H, d), dtype=torch.bfloat16, device="cuda")
    dq, dk, dv = torch.empty_like(o), torch.empty_like(o), torch.empty_like(o)

    def step():
        lib.hstu_jagged_attn_fwd(q, k, v, off, w.max_len, w.alpha, True, out=o, workspace=ws)
        lib.hstu_jagged_attn_bwd(q, k, v, g, off, w.max_len, w.alpha, True, out=(dq, dk, dv), workspace=ws)

    print("graph, large batch", mode, T, flush=True)
    step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for it in range(3):
        print("graph replay, large batch", mode, it, flush=True)
        for t in (q, k, v, g):
            t.copy_(fresh())
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [x.clone() for x in (o, dq, dk, dv)]
        for t in (o, dq, dk, dv):
            t.zero_()
        step()
        torch.cuda.synchronize()
        for name, a, b in zip(("o", "dq", "dk", "dv"), got, (o, dq, dk, dv)):
            assert torch.equal(a, b), (mode, name, it)
            assert torch.isfinite(a.float()).all()
            assert (a != 0).any()
