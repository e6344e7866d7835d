"""The forward entry point that allocates nothing (its scratch is a static device array inside the
library) against the forward that takes a caller's workspace: same kernels, same schedule, so the
outputs must agree bit for bit.  Two calls in a row on the shared array, the second with a smaller
input, and once more after a call that was refused for its size."""
import numpy as np
import pytest
import torch

import paper_2508_04711_amd as lib
import workloads

pytestmark = pytest.mark.gpu


def _batch(name, lengths, heads, d, max_len, seed):
    w = workloads.custom(name, lengths, heads, d, d, max_len, dtype="bf16", seed=seed)
    dev = {k: v.cuda() for k, v in workloads.values(w).items()}
    off = torch.from_numpy(w.seq_offsets()).cuda()
    return w, dev, off


def _both(w, dev, off, out_dtype):
    want = lib.hstu_jagged_attn_fwd(dev["q"], dev["k"], dev["v"], off, w.max_len, w.alpha, True,
                                    out_dtype=out_dtype)
    got = torch.full_like(want, float("nan"))
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    lib.hstu_jagged_attn_fwd_static(dev["q"], dev["k"], dev["v"], off, w.max_len, w.alpha, True, got)
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before  # (torch's allocator, at least)
    torch.cuda.synchronize()
    return want, got


def test_static_scratch_forward_twice_second_smaller():
    assert lib.hstu_static_scratch_bytes() == 16 << 20
    # first: long sequences with ragged tails, several tiles per sequence
    big = _batch("static_a", [1500, 2077, 1101], 2, 128, 2048, 11)
    # second: a smaller batch of short sequences, an empty one among them
    small = _batch("static_b", [130, 0, 1, 77, 300, 64], 2, 128, 300, 12)
    for (w, dev, off), odt in ((big, torch.bfloat16), (small, torch.float32), (big, torch.float32)):
        want, got = _both(w, dev, off, odt)
        assert not torch.isnan(got.float()).any()
        assert torch.equal(want, got), w.name


def test_static_scratch_refuses_what_does_not_fit_and_still_works_after():
    rows = 400_000  # max_len >= 4096: room for the partial results of split tiles, ~900 MB here
    q = torch.empty((rows, 4, 128), dtype=torch.bfloat16, device="cuda")
    off = torch.tensor([0, rows // 2, rows], dtype=torch.int32, device="cuda")
    with pytest.raises(lib.HstuError) as e:
        lib.hstu_jagged_attn_fwd_static(q, q, q, off, 1 << 18, 0.1, True, torch.empty_like(q))
    assert e.value.status == -8
    w, dev, off = _batch("static_c", [257, 33], 4, 64, 257, 13)
    want, got = _both(w, dev, off, torch.bfloat16)
    assert torch.equal(want, got)
