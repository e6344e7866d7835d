"""Pins for the oracle of the attention with timestamp bias (oracle/hstu_oracle_bias.c), CPU only.

The paper does not define the bucket transform, so what is pinned here is that the oracle
computes this build's stated reading correctly: against a dense padded formulation written
with torch (explicit bias matrix, autograd for every gradient including the table's), against
central finite differences, against the unbiased oracle when the table is zero, and the bucket
function against its closed form."""
import numpy as np
import pytest
import torch

import oracle


def _bucket_py(delta, nb, f):
    """The reading, re-derived with Python integers."""
    delta = abs(int(delta))
    if delta <= 1:
        return 0
    e = delta.bit_length() - 1
    top = delta >> (e - f) if e >= f else delta << (f - e)
    return min(nb - 1, e * (1 << f) + top - (1 << f))


def test_bucket_closed_forms():
    for f in (0, 1, 2, 3):
        nb = 31 * (1 << f) + 5
        for e in range(1, 31):
            assert oracle.bias_bucket(1 << e, 0, nb, f) == e * (1 << f)            # powers of two
            assert oracle.bias_bucket(0, 1 << e, nb, f) == e * (1 << f)            # sign does not matter
            if e >= f:                                                             # last group of the octave
                assert oracle.bias_bucket((1 << (e + 1)) - 1, 0, nb, f) == e * (1 << f) + (1 << f) - 1
        assert oracle.bias_bucket(5, 5, nb, f) == 0 and oracle.bias_bucket(6, 5, nb, f) == 0
    rng = np.random.default_rng(0)
    prev = 0
    for d in sorted(int(x) for x in rng.integers(0, 2 ** 31 - 1, size=2000)):
        b = oracle.bias_bucket(d, 0, 128, 2)
        assert b == _bucket_py(d, 128, 2)
        assert b >= prev                       # non-decreasing in the difference
        prev = b
    assert oracle.bias_bucket(2 ** 31 - 1, -(2 ** 31), 40, 2) == 39    # clamps to the last bucket
    # two groups per octave at f = 1: [4,6) and [6,8) are different buckets, [4,5] the same
    assert oracle.bias_bucket(4, 0, 64, 1) == oracle.bias_bucket(5, 0, 64, 1) != oracle.bias_bucket(6, 0, 64, 1)


def _problem(seed, lengths, H, dqk, dv, nb=24, f=1):
    rng = np.random.default_rng(seed)
    off = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    T = int(off[-1])
    q = rng.standard_normal((T, H, dqk)); k = rng.standard_normal((T, H, dqk))
    v = rng.standard_normal((T, H, dv)); g = rng.standard_normal((T, H, dv))
    ts = np.concatenate([np.cumsum(rng.integers(0, 40, size=L)) + rng.integers(0, 1000) for L in lengths]
                        + [np.zeros(0, dtype=np.int64)]).astype(np.int32)
    w = rng.standard_normal(nb)
    return off, q, k, v, g, ts, w, f


def _dense_torch(off, q, k, v, g, ts, w, f, max_len, alpha, causal):
    """Per sequence: dense scores plus an explicit bias matrix, explicit mask, autograd."""
    tq, tk, tv = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (q, k, v))
    tw = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    nb = len(w)
    outs = []
    for b in range(len(off) - 1):
        s, e = int(off[b]), int(off[b + 1])
        L = e - s
        if L == 0:
            continue
        idx = torch.tensor([[_bucket_py(int(ts[s + i]) - int(ts[s + j]), nb, f) for j in range(L)]
                            for i in range(L)], dtype=torch.long)
        bias = tw[idx]                                                   # [L, L]
        sc = torch.einsum("ihd,jhd->hij", tq[s:e], tk[s:e]) + bias[None]
        x = alpha * sc
        mask = torch.tril(torch.ones(L, L, dtype=torch.float64)) if causal else torch.ones(L, L, dtype=torch.float64)
        p = x * torch.sigmoid(x) * mask[None] / max_len
        outs.append(torch.einsum("hij,jhd->ihd", p, tv[s:e]))
    o = torch.cat(outs) if outs else torch.zeros_like(tv)
    loss = (o * torch.tensor(g, dtype=torch.float64)[_rows(off)]).sum()
    loss.backward()
    full = np.zeros_like(v)
    full[_rows(off)] = o.detach().numpy()
    return full, tq.grad.numpy(), tk.grad.numpy(), tv.grad.numpy(), tw.grad.numpy()


def _rows(off):
    return np.concatenate([np.arange(off[b], off[b + 1]) for b in range(len(off) - 1)]).astype(np.int64)


@pytest.mark.parametrize("causal", [True, False])
def test_against_dense_torch_with_explicit_bias_matrix(causal):
    off, q, k, v, g, ts, w, f = _problem(1, [7, 1, 0, 12, 5], 2, 6, 4)
    max_len, alpha = 12, 0.37
    o, dq, dk, dv, dw = oracle.bias_attention(q, k, v, g, off, ts, w, f, max_len, alpha, causal)
    ro, rq, rk, rv, rw = _dense_torch(off, q, k, v, g, ts, w, f, max_len, alpha, causal)
    for name, a, b in (("o", o, ro), ("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv), ("dw", dw, rw)):
        np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-12, err_msg=name)
    assert np.count_nonzero(dw) >= 4            # several buckets are really in use


def test_zero_table_is_the_unbiased_attention():
    off, q, k, v, g, ts, w, f = _problem(2, [9, 3, 14], 2, 5, 7)
    o, dq, dk, dv, dw = oracle.bias_attention(q, k, v, g, off, ts, np.zeros_like(w), f, 14, 0.25, True)
    np.testing.assert_allclose(o, oracle.fwd(q, k, v, off, 14, 0.25, True), rtol=1e-13, atol=1e-15)
    rq, rk, rv = oracle.bwd(q, k, v, g, off, 14, 0.25, True)
    for a, b in ((dq, rq), (dk, rk), (dv, rv)):
        np.testing.assert_allclose(a, b, rtol=1e-13, atol=1e-15)
    assert np.abs(dw).sum() > 0                 # the table still has a gradient at zero


def test_table_gradient_by_finite_differences():
    off, q, k, v, g, ts, w, f = _problem(3, [11, 6], 1, 4, 3, nb=10, f=1)
    max_len, alpha = 11, 0.5
    _, _, _, _, dw = oracle.bias_attention(q, k, v, g, off, ts, w, f, max_len, alpha, True)
    h = 1e-6
    for b in range(len(w)):
        wp, wm = w.copy(), w.copy()
        wp[b] += h; wm[b] -= h
        lp = (oracle.bias_attention(q, k, v, None, off, ts, wp, f, max_len, alpha, True)[0] * g).sum()
        lm = (oracle.bias_attention(q, k, v, None, off, ts, wm, f, max_len, alpha, True)[0] * g).sum()
        assert abs((lp - lm) / (2 * h) - dw[b]) <= 1e-7 * max(1.0, abs(dw[b])), b


def test_constant_table_shifts_every_score():
    # a table with one value c everywhere is the unbiased attention on scores s + c: check one pair
    q = np.array([[[2.0, -1.0]]]); k = np.array([[[0.5, 3.0]]]); v = np.array([[[1.0]]])
    off = np.array([0, 1], dtype=np.int32)
    c = 0.75
    o = oracle.bias_attention(q, k, v, None, off, np.array([5], dtype=np.int32), np.full(8, c), 1, 1, 0.3)[0]
    x = 0.3 * (2.0 * 0.5 - 3.0 + c)
    assert abs(o[0, 0, 0] - x / (1 + np.exp(-x))) < 1e-15


@pytest.mark.parametrize("causal", [True, False])
def test_sampled_rows_equal_the_full_computation(causal):
    """bias_rows (used where the full oracle is too slow) against bias_attention, which the
    tests above pin: every row of a small problem, in shuffled order."""
    off, q, k, v, g, ts, w, f = _problem(11, [9, 1, 23, 0, 14], 2, 5, 3)
    full = oracle.bias_attention(q, k, v, g, off, ts, w, f, 23, 0.37, causal)
    sel = np.random.default_rng(2).permutation(int(off[-1]))
    got = oracle.bias_rows(q, k, v, g, off, ts, w, f, 23, 0.37, causal, sel)
    for name, a, b in zip(("o", "dq", "dk", "dv"), got, full[:4]):
        np.testing.assert_allclose(a, b[sel], rtol=1e-12, atol=1e-14, err_msg=name)
    only_o = oracle.bias_rows(q, k, v, None, off, ts, w, f, 23, 0.37, causal, sel[:5])
    np.testing.assert_allclose(only_o[0], full[0][sel[:5]], rtol=1e-12, atol=1e-14)
    assert only_o[1] is None
    with pytest.raises(Exception):
        oracle.bias_rows(q, k, v, g, off, ts, w, f, 23, 0.37, causal, [int(off[-1])])   # no such row
