"""Calls on a stream other than torch's current one: the outputs and the workspace the binding
allocates must belong to that stream, or the allocator could hand their memory to the current
stream's next allocation while the kernels still use it."""
import pytest
import torch

import workloads

pytestmark = pytest.mark.gpu


def test_side_stream_calls_keep_their_temporaries_while_the_current_stream_allocates():
    import paper_2508_04711_amd as lib
    # several tiles per sequence
    w = workloads.custom("side_stream", [1500, 2077, 1201], 2, 128, 128, 2077, dtype="bf16", seed=21)
    dev = {k: v.cuda() for k, v in workloads.values(w).items()}
    off = torch.from_numpy(w.seq_offsets()).cuda()
    args = (dev["q"], dev["k"], dev["v"])
    ref_o = lib.hstu_jagged_attn_fwd(*args, off, w.max_len, w.alpha, True)
    ref_g = lib.hstu_jagged_attn_bwd(*args, dev["d_o"], off, w.max_len, w.alpha, True)
    torch.cuda.synchronize()
    p = (len(w.lengths), w.num_heads, w.d_qk, w.d_v, w.max_len, w.alpha, True, 0, w.total_rows)
    sizes = [lib.hstu_jagged_attn_workspace_bytes(p, 0), lib.hstu_jagged_attn_workspace_bytes(p, 1),
             dev["q"].numel() * 2]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    outs = []
    for rep in range(4):
        o = lib.hstu_jagged_attn_fwd(*args, off, w.max_len, w.alpha, True, stream=side)
        g = lib.hstu_jagged_attn_bwd(*args, dev["d_o"], off, w.max_len, w.alpha, True, stream=side)
        outs.append((o, g))
        # meanwhile the current stream allocates blocks of the same sizes and overwrites them
        junk = [torch.empty(n, dtype=torch.uint8, device="cuda").fill_(0xFF) for n in sizes for _ in range(2)]
        del junk
    side.synchronize()
    torch.cuda.synchronize()
    for o, g in outs:
        assert torch.equal(o, ref_o)
        for got, want in zip(g, ref_g):
            assert torch.equal(got, want)
