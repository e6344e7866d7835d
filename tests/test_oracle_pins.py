"""Pins for the CPU oracle: each test ties it to something other than itself.

The oracle (oracle/hstu_oracle.c) is the definition of the paper's section 2.1
equation written out pair by pair.  Here it is checked against
  * an independently structured dense, padded, explicitly masked einsum,
  * torch autograd and central finite differences for the gradients,
  * closed forms (constant scores, zero queries, length-one sequences),
  * textbook values of SiLU,
  * structural invariants (prefix property, linearity, batch composition),
  * the hand-worked chunk ownership table of section 2.3 and the
    "partials add up to full attention" identity.
All of it runs on the CPU.
"""
import os

import numpy as np
import pytest
import torch

import oracle

RNG = np.random.default_rng(1234)


def _batch(lengths, H, dqk, dv, seed=0, scale=1.0):
    rng = np.random.default_rng(seed)
    T = int(sum(lengths))
    off = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    q = rng.normal(size=(T, H, dqk)) * scale
    k = rng.normal(size=(T, H, dqk)) * scale
    v = rng.normal(size=(T, H, dv)) * scale
    d_o = rng.normal(size=(T, H, dv)) * scale
    return off, q, k, v, d_o


def _dense_fwd(q, k, v, off, N, alpha, causal):
    """Pad every sequence to Lmax, score all pairs, mask explicitly (independent of the oracle)."""
    B = len(off) - 1
    lens = np.diff(off)
    Lm = int(lens.max()) if B else 0
    T, H, dqk = q.shape
    dv = v.shape[2]
    qp = np.zeros((B, Lm, H, dqk)); kp = np.zeros((B, Lm, H, dqk)); vp = np.zeros((B, Lm, H, dv))
    for b in range(B):
        qp[b, :lens[b]] = q[off[b]:off[b + 1]]
        kp[b, :lens[b]] = k[off[b]:off[b + 1]]
        vp[b, :lens[b]] = v[off[b]:off[b + 1]]
    s = np.einsum("bihd,bjhd->bhij", qp, kp) * alpha
    p = s / (1.0 + np.exp(-s))
    i = np.arange(Lm)[:, None]
    j = np.arange(Lm)[None, :]
    mask = np.ones((B, 1, Lm, Lm), dtype=bool)
    if causal:
        mask &= (j <= i)[None, None]
    valid = np.arange(Lm)[None, :] < lens[:, None]               # [B, Lm]
    mask = mask & valid[:, None, :, None] & valid[:, None, None, :]
    p = np.where(mask, p, 0.0)
    op = np.einsum("bhij,bjhd->bihd", p, vp) / N
    o = np.zeros((T, H, dv))
    for b in range(B):
        o[off[b]:off[b + 1]] = op[b, :lens[b]]
    return o


def _torch_dense_grads(q, k, v, d_o, off, N, alpha, causal):
    """Gradients from torch autograd through a per-sequence dense formulation."""
    tq = torch.tensor(q, dtype=torch.float64, requires_grad=True)
    tk = torch.tensor(k, dtype=torch.float64, requires_grad=True)
    tv = torch.tensor(v, dtype=torch.float64, requires_grad=True)
    tdo = torch.tensor(d_o, dtype=torch.float64)
    loss = 0.0
    for b in range(len(off) - 1):
        s, e = int(off[b]), int(off[b + 1])
        if e == s:
            continue
        sc = torch.einsum("ihd,jhd->hij", tq[s:e], tk[s:e]) * alpha
        p = torch.nn.functional.silu(sc)
        if causal:
            p = torch.tril(p)
        o = torch.einsum("hij,jhd->ihd", p, tv[s:e]) / N
        loss = loss + (o * tdo[s:e]).sum()
    loss.backward()
    return tq.grad.numpy(), tk.grad.numpy(), tv.grad.numpy()


# --- forward against the dense masked definition --------------------------------------------

@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("lengths,H,dqk,dv", [
    ([5, 1, 7, 3], 2, 4, 3),
    ([1], 1, 2, 2),
    ([9, 0, 4], 3, 8, 5),          # an empty sequence in the middle
    ([55, 41, 33, 18], 2, 32, 32),  # the tiny benchmark configuration's shape
])
def test_fwd_matches_dense_masked_einsum(lengths, H, dqk, dv, causal):
    off, q, k, v, _ = _batch(lengths, H, dqk, dv, seed=len(lengths))
    N, alpha = 64, 1.0 / np.sqrt(dqk)
    got = oracle.fwd(q, k, v, off, N, alpha, causal)
    want = _dense_fwd(q, k, v, off, N, alpha, causal)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)


# --- gradients -------------------------------------------------------------------------------

@pytest.mark.parametrize("causal", [True, False])
def test_bwd_matches_torch_autograd(causal):
    off, q, k, v, d_o = _batch([6, 1, 11, 0, 4], 2, 5, 3, seed=7)
    N, alpha = 16, 0.37
    dq, dk, dv = oracle.bwd(q, k, v, d_o, off, N, alpha, causal)
    rq, rk, rv = _torch_dense_grads(q, k, v, d_o, off, N, alpha, causal)
    np.testing.assert_allclose(dq, rq, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(dk, rk, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(dv, rv, rtol=1e-11, atol=1e-13)


def test_bwd_matches_central_finite_differences():
    off, q, k, v, d_o = _batch([4, 1, 6], 2, 3, 2, seed=3)
    N, alpha, causal = 8, 0.5, True
    dq, dk, dv = oracle.bwd(q, k, v, d_o, off, N, alpha, causal)

    def loss(q_, k_, v_):
        return float((oracle.fwd(q_, k_, v_, off, N, alpha, causal) * d_o).sum())

    h = 1e-6
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        fd = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            xp = x.copy(); xm = x.copy()
            xp[idx] += h; xm[idx] -= h
            args_p = {"q": q, "k": k, "v": v}; args_m = dict(args_p)
            args_p[name] = xp; args_m[name] = xm
            fd[idx] = (loss(args_p["q"], args_p["k"], args_p["v"])
                       - loss(args_m["q"], args_m["k"], args_m["v"])) / (2 * h)
        np.testing.assert_allclose(g, fd, rtol=2e-6, atol=1e-8, err_msg="d" + name)


# --- closed forms ----------------------------------------------------------------------------

def test_constant_scores_give_scaled_prefix_sums():
    # Q = K = sqrt(c/alpha) * e1  =>  alpha*<q,k> = c for every pair, so
    # O[i] = silu(c)/N * (V[0] + ... + V[i]): diagonal included, 1/N applied once.
    L, H, d, dv = 9, 2, 4, 3
    N, alpha, c = 10, 0.25, 1.0
    off = np.array([0, L], dtype=np.int32)
    q = np.zeros((L, H, d)); q[:, :, 0] = np.sqrt(c / alpha)
    k = q.copy()
    v = np.random.default_rng(5).normal(size=(L, H, dv))
    got = oracle.fwd(q, k, v, off, N, alpha, True)
    silu1 = 0.7310585786300049          # 1/(1+e^-1)
    want = silu1 / N * np.cumsum(v, axis=0)
    np.testing.assert_allclose(got, want, rtol=1e-13)
    got_nc = oracle.fwd(q, k, v, off, N, alpha, False)
    want_nc = np.broadcast_to(silu1 / N * v.sum(axis=0, keepdims=True), v.shape)
    np.testing.assert_allclose(got_nc, want_nc, rtol=1e-13)


def test_zero_queries():
    # silu(0) = 0 => O = 0, dV = 0 exactly; silu'(0) = 1/2 =>
    # dQ[i] = alpha/(2N) * sum_{j<=i} <dO[i],V[j]> K[j]; dK[j] = alpha/(2N) * sum_i (..) Q[i] = 0.
    off, q, k, v, d_o = _batch([7, 3], 2, 4, 5, seed=11)
    q[:] = 0.0
    N, alpha = 12, 0.3
    o = oracle.fwd(q, k, v, off, N, alpha, True)
    dq, dk, dv = oracle.bwd(q, k, v, d_o, off, N, alpha, True)
    assert np.all(o == 0.0) and np.all(dv == 0.0) and np.all(dk == 0.0)
    want = np.zeros_like(dq)
    for b in range(2):
        s, e = off[b], off[b + 1]
        for h in range(2):
            g = np.tril(d_o[s:e, h] @ v[s:e, h].T)           # <dO[i],V[j]> for j <= i
            want[s:e, h] = alpha / (2 * N) * g @ k[s:e, h]
    np.testing.assert_allclose(dq, want, rtol=1e-12, atol=1e-15)


def test_length_one_sequences_scalar_closed_form():
    B, H, d, dv = 3, 2, 4, 3
    off, q, k, v, d_o = _batch([1] * B, H, d, dv, seed=13)
    N, alpha = 5, 0.7
    o = oracle.fwd(q, k, v, off, N, alpha, True)
    dq, dk, dvv = oracle.bwd(q, k, v, d_o, off, N, alpha, True)
    x = alpha * (q * k).sum(-1, keepdims=True)
    sg = 1 / (1 + np.exp(-x))
    np.testing.assert_allclose(o, x * sg / N * v, rtol=1e-13)
    ds = (d_o * v).sum(-1, keepdims=True) / N * sg * (1 + x * (1 - sg))
    np.testing.assert_allclose(dq, alpha * ds * k, rtol=1e-12)
    np.testing.assert_allclose(dk, alpha * ds * q, rtol=1e-12)
    np.testing.assert_allclose(dvv, x * sg / N * d_o, rtol=1e-12)


def test_silu_textbook_values():
    assert oracle.silu(0.0) == 0.0
    assert abs(oracle.silu(1.0) - 0.7310585786300049) < 1e-15
    assert abs(oracle.silu_grad(0.0) - 0.5) < 1e-15
    # the global minimum of x*sigmoid(x): value -0.27846..., at x = -1.27846...
    xs = np.linspace(-1.3, -1.25, 5001)
    vals = np.array([oracle.silu(x) for x in xs])
    assert abs(vals.min() + 0.2784645427610738) < 1e-9
    assert abs(xs[vals.argmin()] + 1.2784645427610738) < 2e-5
    assert abs(oracle.silu_grad(-1.2784645427610738)) < 1e-9
    # asymptotes and no overflow
    for x in (800.0, -800.0, 1e4, -1e4):
        s, g = oracle.silu(x), oracle.silu_grad(x)
        assert np.isfinite(s) and np.isfinite(g)
    assert oracle.silu(800.0) == 800.0 and abs(oracle.silu(-800.0)) < 1e-300
    assert abs(oracle.silu_grad(800.0) - 1.0) < 1e-12 and abs(oracle.silu_grad(-800.0)) < 1e-300


def test_scale_sits_inside_silu_and_mask_outside():
    # One query, one key: O = silu(alpha*s)/N * v, which differs from alpha*silu(s)/N * v.
    off = np.array([0, 1], dtype=np.int32)
    q = np.array([[[2.0, 0.0]]]); k = np.array([[[3.0, 0.0]]]); v = np.array([[[1.0]]])
    o = oracle.fwd(q, k, v, off, 1, 0.5, True)
    assert abs(o[0, 0, 0] - 3.0 / (1 + np.exp(-3.0))) < 1e-14
    # masked pairs contribute exactly zero even when silu of their score is not zero
    off2 = np.array([0, 2], dtype=np.int32)
    q2 = np.array([[[1.0]], [[1.0]]]); k2 = np.array([[[1.0]], [[5.0]]]); v2 = np.array([[[1.0]], [[100.0]]])
    o2 = oracle.fwd(q2, k2, v2, off2, 1, 1.0, True)
    assert abs(o2[0, 0, 0] - 1.0 / (1 + np.exp(-1.0))) < 1e-14


# --- invariants ------------------------------------------------------------------------------

def test_causal_prefix_property():
    off, q, k, v, d_o = _batch([13], 2, 6, 4, seed=17)
    N, alpha, m = 13, 0.4, 8
    full = oracle.fwd(q, k, v, off, N, alpha, True)
    offm = np.array([0, m], dtype=np.int32)
    part = oracle.fwd(q[:m], k[:m], v[:m], offm, N, alpha, True)
    assert np.array_equal(full[:m], part)
    # gradients from a dO that is zero beyond row m equal those of the truncated problem
    d_o_t = d_o.copy(); d_o_t[m:] = 0.0
    dq, dk, dv = oracle.bwd(q, k, v, d_o_t, off, N, alpha, True)
    dq2, dk2, dv2 = oracle.bwd(q[:m], k[:m], v[:m], d_o[:m], offm, N, alpha, True)
    np.testing.assert_allclose(dq[:m], dq2, rtol=1e-13, atol=1e-16)
    np.testing.assert_allclose(dk[:m], dk2, rtol=1e-13, atol=1e-16)
    np.testing.assert_allclose(dv[:m], dv2, rtol=1e-13, atol=1e-16)
    assert np.all(dq[m:] == 0) and np.all(dk[m:] == 0) and np.all(dv[m:] == 0)


def test_linearity_in_v_and_in_one_over_n():
    off, q, k, v, _ = _batch([6, 9], 2, 4, 4, seed=19)
    v2 = np.random.default_rng(23).normal(size=v.shape)
    a = oracle.fwd(q, k, v, off, 7, 0.5, True)
    b = oracle.fwd(q, k, v2, off, 7, 0.5, True)
    c = oracle.fwd(q, k, v + v2, off, 7, 0.5, True)
    np.testing.assert_allclose(c, a + b, rtol=1e-12, atol=1e-14)
    d = oracle.fwd(q, k, v, off, 14, 0.5, True)
    np.testing.assert_allclose(d, a / 2, rtol=1e-14)
    # max_len = 1 is the equation exactly as printed (no normaliser)
    e = oracle.fwd(q, k, v, off, 1, 0.5, True)
    np.testing.assert_allclose(e, a * 7, rtol=1e-14)


def test_batch_composition_invariance():
    lengths = [5, 12, 1, 8]
    off, q, k, v, d_o = _batch(lengths, 2, 4, 4, seed=29)
    N, alpha = 12, 0.5
    o = oracle.fwd(q, k, v, off, N, alpha, True)
    dq, dk, dv = oracle.bwd(q, k, v, d_o, off, N, alpha, True)
    for b, L in enumerate(lengths):
        s, e = off[b], off[b + 1]
        o1 = oracle.fwd(q[s:e], k[s:e], v[s:e], [0, L], N, alpha, True)
        g1 = oracle.bwd(q[s:e], k[s:e], v[s:e], d_o[s:e], [0, L], N, alpha, True)
        assert np.array_equal(o[s:e], o1)
        for full, alone in zip((dq, dk, dv), g1):
            assert np.array_equal(full[s:e], alone)


def test_noncausal_equal_lengths_is_two_gemms():
    L, d, dv = 10, 6, 5
    off, q, k, v, _ = _batch([L], 1, d, dv, seed=31)
    N, alpha = 3, 0.2
    s = alpha * (q[:, 0] @ k[:, 0].T)
    want = (s / (1 + np.exp(-s))) @ v[:, 0] / N
    got = oracle.fwd(q, k, v, off, N, alpha, False)
    np.testing.assert_allclose(got[:, 0], want, rtol=1e-12, atol=1e-15)


def test_sampled_rows_equal_full_results():
    off, q, k, v, d_o = _batch([17, 2, 30], 2, 8, 4, seed=37)
    N, alpha = 32, 0.35
    o = oracle.fwd(q, k, v, off, N, alpha, True)
    dq, dk, dv = oracle.bwd(q, k, v, d_o, off, N, alpha, True)
    sel = [0, 16, 17, 18, 19, 48, 30]
    so, sdq, sdk, sdv = oracle.rows(q, k, v, d_o, off, N, alpha, True, sel)
    assert np.array_equal(so, o[sel]) and np.array_equal(sdq, dq[sel])
    assert np.array_equal(sdk, dk[sel]) and np.array_equal(sdv, dv[sel])
    only_o = oracle.rows(q, k, v, None, off, N, alpha, True, sel)
    assert np.array_equal(only_o, o[sel])


# --- context-parallel split ------------------------------------------------------------------

def _golden_chunks():
    path = os.path.join(os.path.dirname(__file__), "golden", "cp_chunks.txt")
    rows = []
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        head, tail = line.split(":")
        L, cp, rank = (int(x) for x in head.split())
        rows.append((L, cp, rank, [int(x) for x in tail.split()]))
    return rows


def test_chunk_ownership_matches_hand_worked_table():
    for L, cp, rank, want in _golden_chunks():
        seq, pos = oracle.cp_local_map([0, L], cp, rank)
        assert list(pos) == want, (L, cp, rank)
        assert np.all(seq == 0)


def test_chunk_ownership_partitions_every_sequence():
    lengths = [16, 5, 0, 23, 1, 40]
    off = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    for cp in (1, 2, 3, 4, 8):
        seen = np.concatenate([oracle.cp_global_rows(off, cp, r) for r in range(cp)])
        assert sorted(seen.tolist()) == list(range(off[-1]))


def test_balanced_visible_pairs_per_rank():
    # With 2*CP | L and chunk size c, rank r sees (r*c^2 + c(c+1)/2) pairs from its first
    # chunk and ((2CP-1-r)*c^2 + c(c+1)/2) from its second: 2*CP*c^2 - c^2 + c(c+1) in all,
    # the same for every rank.
    for L, cp in ((16, 2), (48, 4), (64, 8), (24, 1)):
        c = L // (2 * cp)
        want = (2 * cp - 1) * c * c + c * (c + 1)
        for r in range(cp):
            _, pos = oracle.cp_local_map([0, L], cp, r)
            pairs = int(sum(p + 1 for p in pos))      # causal: position p sees p+1 keys
            assert pairs == want, (L, cp, r)
        assert want * cp == L * (L + 1) // 2


@pytest.mark.parametrize("cp", [1, 2, 4])
@pytest.mark.parametrize("causal", [True, False])
def test_partials_add_up_to_full_attention(cp, causal):
    lengths = [16, 5, 23, 1, 0, 32]
    off, q, k, v, d_o = _batch(lengths, 2, 4, 3, seed=41)
    N, alpha = 32, 0.45
    o = oracle.fwd(q, k, v, off, N, alpha, causal)
    dq, dk, dv = oracle.bwd(q, k, v, d_o, off, N, alpha, causal)
    rows = [oracle.cp_global_rows(off, cp, r) for r in range(cp)]
    o_sum = np.zeros_like(o); dq_sum = np.zeros_like(dq)
    dk_sum = np.zeros_like(dk); dv_sum = np.zeros_like(dv)
    for rq in range(cp):
        gq = rows[rq]
        # against every key at once (kv_rank = -1) ...
        o_all, dq_all, dk_all, dv_all = oracle.cp_partial(
            q[gq], k, v, d_o[gq], off, N, alpha, causal, cp, rq, -1)
        np.testing.assert_allclose(o_all, o[gq], rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(dq_all, dq[gq], rtol=1e-12, atol=1e-15)
        dk_sum += dk_all; dv_sum += dv_all
        # ... and one key rank at a time: the pieces add up
        o_acc = np.zeros_like(o_all); dq_acc = np.zeros_like(dq_all)
        for rk in range(cp):
            gk = rows[rk]
            po, pdq, pdk, pdv = oracle.cp_partial(
                q[gq], k[gk], v[gk], d_o[gq], off, N, alpha, causal, cp, rq, rk)
            o_acc += po; dq_acc += pdq
        np.testing.assert_allclose(o_acc, o[gq], rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(dq_acc, dq[gq], rtol=1e-12, atol=1e-15)
        o_sum[gq] = o_acc; dq_sum[gq] = dq_acc
    np.testing.assert_allclose(o_sum, o, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(dk_sum, dk, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(dv_sum, dv, rtol=1e-12, atol=1e-15)
    # dK/dV of one key part = sum over query ranks of the per-pair partials
    for rk in range(cp):
        gk = rows[rk]
        dk_acc = np.zeros((len(gk),) + dk.shape[1:]); dv_acc = np.zeros((len(gk),) + dv.shape[1:])
        for rq in range(cp):
            gq = rows[rq]
            _, _, pdk, pdv = oracle.cp_partial(
                q[gq], k[gk], v[gk], d_o[gq], off, N, alpha, causal, cp, rq, rk)
            dk_acc += pdk; dv_acc += pdv
        np.testing.assert_allclose(dk_acc, dk[gk], rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(dv_acc, dv[gk], rtol=1e-12, atol=1e-15)


def test_cp_partial_selected_rows_equal_full_partial():
    off, q, k, v, d_o = _batch([24, 9, 40], 2, 4, 4, seed=43)
    cp, rq, rk, N, alpha = 2, 1, 0, 40, 0.5
    gq, gk = oracle.cp_global_rows(off, cp, rq), oracle.cp_global_rows(off, cp, rk)
    full = oracle.cp_partial(q[gq], k[gk], v[gk], d_o[gq], off, N, alpha, True, cp, rq, rk)
    sq, sk = [0, 5, len(gq) - 1], [1, len(gk) - 1]
    part = oracle.cp_partial(q[gq], k[gk], v[gk], d_o[gq], off, N, alpha, True, cp, rq, rk,
                             sel_q=sq, sel_k=sk)
    assert np.array_equal(part[0][sq], full[0][sq]) and np.array_equal(part[1][sq], full[1][sq])
    assert np.array_equal(part[2][sk], full[2][sk]) and np.array_equal(part[3][sk], full[3][sk])
