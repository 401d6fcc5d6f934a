"""Pins of the oracle's backward pass and row statistics (CPU only).

The paper gives no gradient (Sec. 4.3-4.4 train through the method without describing it); the
oracle differentiates the forward with every Q block's grouping held fixed. What fixes it here:
  * finite differences of the oracle's own *forward* (Richardson-extrapolated central
    differences on dyadic inputs, exact perturbations),
  * automatic differentiation (torch, float64) of a restatement of Eq. 2 by index_select / sum
    whose forward value is first checked against the oracle's forward,
  * one column per group = exact attention, whose gradient torch's own attention gives,
  * the structure the reading implies (unsampled Q columns get no gradient, the members of a
    K group get the same one).
"""
import numpy as np
import pytest
import torch

import oracle


def dyadic(rng, shape, span=2.0, step=1 / 64):
    """Multiples of `step` in [-span, span]: perturbations by 2^-9 stay exact in float32."""
    n = int(span / step)
    return (rng.integers(-n, n + 1, size=shape) * step).astype(np.float32)


def problem(seed, B=1, H=2, Hkv=1, N=24, Nk=None, d=16, Br=8, n_groups=8, causal=False, scale=None):
    rng = np.random.default_rng(seed)
    Nk_ = N if Nk is None else Nk
    q = dyadic(rng, (B, H, N, d))
    k = dyadic(rng, (B, Hkv, Nk_, d))
    v = dyadic(rng, (B, Hkv, Nk_, d))
    do = dyadic(rng, (B, H, N, d))
    p = oracle.params(B, H, Hkv, N, d, Br, n_groups, causal=causal, n_planes=8, lsh_seed=seed, scale=scale, Nk=Nk)
    return q, k, v, do, p


def mask_of(N, Nk, causal):
    if not causal:
        return torch.ones(N, Nk, dtype=torch.bool)
    i = torch.arange(N)[:, None]
    n = torch.arange(Nk)[None, :]
    return n <= i + (Nk - N)


def torch_forward(q, k, v, p, perm):
    """Eq. 2 per Q block with tensor ops: gather the sampled Q columns, sum the grouped K columns."""
    B, H, N, d = q.shape
    Nk = k.shape[2]
    rep = H // k.shape[1]
    G = d // p.n_groups
    mask = mask_of(N, Nk, p.causal)
    out = []
    for b in range(B):
        for h in range(H):
            rows = []
            for t in range((N + p.Br - 1) // p.Br):
                r0, r1 = t * p.Br, min(N, (t + 1) * p.Br)
                pm = torch.as_tensor(perm[b, h, t].astype(np.int64))
                q_r = q[b, h, r0:r1].index_select(1, pm[::G])
                k_f = k[b, h // rep].index_select(1, pm).reshape(Nk, p.n_groups, G).sum(-1)
                s = p.scale * q_r @ k_f.T
                s = s.masked_fill(~mask[r0:r1], float("-inf"))
                rows.append(torch.softmax(s, -1) @ v[b, h // rep])
            out.append(torch.cat(rows))
    return torch.stack(out).reshape(B, H, N, d)


CASES = [dict(), dict(causal=True), dict(H=4, Hkv=2, N=20, Nk=29, causal=True), dict(N=17, Nk=9, Br=4, d=8, n_groups=2),
         dict(B=2, N=30, Br=16, d=32, n_groups=8, scale=0.5)]


@pytest.mark.parametrize("kw", CASES)
def test_distr_backward_matches_automatic_differentiation(kw):
    q, k, v, do, p = problem(11, **kw)
    _, perm, _ = oracle.lsh_group(q, p)
    tq, tk, tv = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (q, k, v))
    o = torch_forward(tq, tk, tv, p, perm)
    assert np.abs(o.detach().numpy() - oracle.distr_fwd(q, k, v, p)).max() < 1e-12
    (o * torch.tensor(do, dtype=torch.float64)).sum().backward()
    dq, dk, dv = oracle.distr_bwd(q, k, v, do, p)
    for got, ref in ((dq, tq.grad), (dk, tk.grad), (dv, tv.grad)):
        assert np.abs(got - ref.numpy()).max() < 1e-11
    # a caller's table gives the same as the LSH stage that produced it
    for a, b_ in zip(oracle.distr_bwd(q, k, v, do, p, perm=perm), (dq, dk, dv)):
        assert np.array_equal(a, b_)


@pytest.mark.parametrize("kw", [dict(), dict(causal=True), dict(H=6, Hkv=2, N=13, Nk=31, causal=True), dict(N=21, Nk=5)])
def test_exact_backward_matches_library_attention(kw):
    q, k, v, do, p = problem(5, **kw)
    tq, tk, tv = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (q, k, v))
    rep = q.shape[1] // k.shape[1]
    o = torch.nn.functional.scaled_dot_product_attention(
        tq, tk.repeat_interleave(rep, 1), tv.repeat_interleave(rep, 1),
        attn_mask=mask_of(p.N, oracle.n_keys(p), p.causal), scale=p.scale)
    (o * torch.tensor(do, dtype=torch.float64)).sum().backward()
    dq, dk, dv = oracle.exact_bwd(q, k, v, do, p)
    for got, ref in ((dq, tq.grad), (dk, tk.grad), (dv, tv.grad)):
        assert np.abs(got - ref.numpy()).max() < 1e-11
    # one column per group (Sec. 3.1): the approximation's gradient is the exact one
    p1 = oracle.params(p.B, p.H, p.Hkv, p.N, p.d, p.Br, p.d, causal=p.causal, n_planes=8, scale=p.scale, Nk=p.Nk)
    for a, b_ in zip(oracle.distr_bwd(q, k, v, do, p1), (dq, dk, dv)):
        assert np.abs(a - b_).max() < 1e-12


@pytest.mark.parametrize("causal", [False, True])
def test_backward_is_the_finite_difference_of_the_forward(causal):
    q, k, v, do, p = problem(23, N=16, Nk=20, Br=8, d=16, n_groups=4, causal=causal)
    _, perm, _ = oracle.lsh_group(q, p)

    def loss(q_, k_, v_):
        return float((oracle.distr_fwd(q_, k_, v_, p, perm=perm) * do).sum())

    def richardson(arrs, which, idx):
        vals = []
        for hstep in (2.0 ** -8, 2.0 ** -9):
            lo = [a.copy() for a in arrs]
            hi = [a.copy() for a in arrs]
            lo[which][idx] -= hstep
            hi[which][idx] += hstep
            assert hi[which][idx] - arrs[which][idx] == hstep    # exact in float32
            vals.append((loss(*hi) - loss(*lo)) / (2 * hstep))
        return (4 * vals[1] - vals[0]) / 3

    grads = oracle.distr_bwd(q, k, v, do, p, perm=perm)
    rng = np.random.default_rng(0)
    scale_of = max(np.abs(g).max() for g in grads)
    for which, arr in enumerate((q, k, v)):
        for _ in range(12):
            idx = tuple(int(rng.integers(0, s)) for s in arr.shape)
            fd = richardson([q, k, v], which, idx)
            assert abs(fd - grads[which][idx]) < 1e-7 * scale_of, (which, idx, fd, grads[which][idx])
    # with the LSH stage live, the same holds wherever the perturbation leaves the table alone
    # (it is piecewise constant in Q); count that such points are the rule, not the exception
    live = oracle.distr_bwd(q, k, v, do, p)
    assert all(np.array_equal(a, b_) for a, b_ in zip(live, grads))
    unchanged = 0
    for _ in range(12):
        idx = tuple(int(rng.integers(0, s)) for s in q.shape)
        tables = []
        for sgn in (-1, 1):
            q2 = q.copy()
            q2[idx] += sgn * 2.0 ** -8
            tables.append(oracle.lsh_group(q2, p)[1])
        if all(np.array_equal(t, perm) for t in tables):
            unchanged += 1
            lo, hi = q.copy(), q.copy()
            lo[idx] -= 2.0 ** -8
            hi[idx] += 2.0 ** -8
            fd = float(((oracle.distr_fwd(hi, k, v, p) - oracle.distr_fwd(lo, k, v, p)) * do).sum()) / 2.0 ** -7
            assert abs(fd - grads[0][idx]) < 1e-3 * scale_of
    assert unchanged >= 8


def test_structure_of_the_gradient():
    q, k, v, do, p = problem(3, H=1, N=8, Nk=12, Br=8, d=16, n_groups=4)
    _, perm, _ = oracle.lsh_group(q, p)
    dq, dk, dv = oracle.distr_bwd(q, k, v, do, p)
    G = p.d // p.n_groups
    pm = perm[0, 0, 0]
    sampled = set(int(c) for c in pm[::G])
    for c in range(p.d):
        if c in sampled:
            assert np.abs(dq[0, 0, :, c]).max() > 0
        else:
            assert np.all(dq[0, 0, :, c] == 0)
    for j in range(p.n_groups):          # one Q block: the members of a K group share one gradient
        cols = dk[0, 0][:, pm[j * G:(j + 1) * G].astype(int)]
        assert np.abs(cols - cols[:, :1]).max() < 1e-15
    # dV does not depend on which V is used beyond P: it is P^T dO with P of the forward
    s_hat, _ = oracle.scores(q, k, p, want_exact=False)
    P = np.exp(s_hat - s_hat.max(1, keepdims=True))
    P /= P.sum(1, keepdims=True)
    assert np.abs(dv[0, 0] - P.T @ do[0, 0].astype(np.float64)).max() < 1e-13


@pytest.mark.parametrize("kw", CASES)
def test_distr_backward_is_the_exact_backward_on_the_replicated_queries(kw):
    """S^ = Q_r K_f^T = Q~ K^T with Q~ = Q whose every channel is replaced by the sampled channel
    of its group (a sum over groups of sums over members): the gradient with the grouping held
    fixed is the exact-attention gradient taken at Q~, with dQ~ summed over each group's members
    into the sampled channel. The matrix-core kernels compute it that way; here the two oracle
    functions are held against each other."""
    q, k, v, do, p = problem(21, **kw)
    _, perm, _ = oracle.lsh_group(q, p)
    G = p.d // p.n_groups
    q_rep = np.empty_like(q)
    Tq = (p.N + p.Br - 1) // p.Br
    for b in range(p.B):
        for h in range(p.H):
            for t in range(Tq):
                rows = slice(t * p.Br, min(p.N, (t + 1) * p.Br))
                pm = perm[b, h, t].astype(int)
                for j in range(p.n_groups):
                    for c in pm[j * G:(j + 1) * G]:
                        q_rep[b, h, rows, c] = q[b, h, rows, pm[j * G]]
    p_exact = oracle.params(p.B, p.H, p.Hkv, p.N, p.d, p.Br, p.d, causal=bool(p.causal), scale=p.scale,
                            Nk=p.Nk if p.Nk > 0 else None)
    assert np.abs(oracle.exact_fwd(q_rep, k, v, p_exact) - oracle.distr_fwd(q, k, v, p)).max() < 1e-12
    dq_rep, dk_e, dv_e = oracle.exact_bwd(q_rep, k, v, do, p_exact)
    dq, dk, dv = oracle.distr_bwd(q, k, v, do, p)
    dq_sum = np.zeros_like(dq)
    for b in range(p.B):
        for h in range(p.H):
            for t in range(Tq):
                rows = slice(t * p.Br, min(p.N, (t + 1) * p.Br))
                pm = perm[b, h, t].astype(int)
                for j in range(p.n_groups):
                    dq_sum[b, h, rows, pm[j * G]] = dq_rep[b, h, rows][:, pm[j * G:(j + 1) * G]].sum(-1)
    unit = max(1.0, np.abs(dq).max(), np.abs(dk).max())
    assert np.abs(dq_sum - dq).max() < 1e-12 * unit
    assert np.abs(dk_e - dk).max() < 1e-12 * unit
    assert np.abs(dv_e - dv).max() < 1e-12 * unit


@pytest.mark.parametrize("kw", [dict(), dict(causal=True, N=20, Nk=29), dict(H=4, Hkv=2, causal=True)])
def test_row_statistics(kw):
    q, k, v, do, p = problem(9, **kw)
    rep = p.H // p.Hkv
    mask = mask_of(p.N, oracle.n_keys(p), p.causal)
    for distr in (True, False):
        got = oracle.lse(q, k, p, distr=distr)
        for b in range(p.B):
            for h in range(p.H):
                s_hat, s = oracle.scores(q, k, p, b=b, h=h)
                s_t = torch.tensor(s_hat if distr else s).masked_fill(~mask, float("-inf"))
                assert np.abs(got[b, h] - torch.logsumexp(s_t, -1).numpy()).max() < 1e-12
    del rep, v, do


def test_bad_arguments():
    q, k, v, do, p = problem(1)
    bad = oracle.params(p.B, p.H, p.Hkv, p.N, p.d, p.Br, 5, n_planes=8)     # 16 % 5 != 0
    with pytest.raises(ValueError):
        oracle.distr_bwd(q, k, v, do, bad)
    mirrored = oracle.params(p.B, p.H, p.Hkv, p.N, p.d, p.Br, p.n_groups, n_planes=8, side=1, Bc=8)
    with pytest.raises(ValueError):
        oracle.distr_bwd(q, k, v, do, mirrored)
