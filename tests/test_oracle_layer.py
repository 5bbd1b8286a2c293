"""Pins for the oracle's dispatch, expert FFN, combine and the whole layer,
forward and backward.

Independent references used: naive Python loops, torch's fp64 gelu/relu and
autograd (a library differentiator, applied to a forward written separately in
torch), central finite differences, adjoint identities and closed forms.
"""
import math

import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2109_10465_amd import inputs as I


def rnd(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- activation
def test_activations_against_torch_and_closed_forms():
    z = np.linspace(-6, 6, 241)
    zt = torch.tensor(z, dtype=torch.float64, requires_grad=True)
    g = torch.nn.functional.gelu(zt)                 # exact erf form
    np.testing.assert_allclose(O.act(z, O.GELU), g.detach().numpy(), rtol=1e-12, atol=1e-15)
    g.sum().backward()
    np.testing.assert_allclose(O.act_grad(z, O.GELU), zt.grad.numpy(), rtol=1e-11, atol=1e-14)
    assert O.act(np.array([0.0]), O.GELU)[0] == 0.0
    assert O.act_grad(np.array([0.0]), O.GELU)[0] == 0.5
    assert O.act(np.array([1.0]), O.GELU)[0] == pytest.approx(0.5 * (1 + math.erf(1 / math.sqrt(2))))
    assert O.act(np.array([30.0]), O.GELU)[0] == 30.0 and abs(O.act(np.array([-30.0]), O.GELU)[0]) < 1e-100
    np.testing.assert_array_equal(O.act(z, O.RELU), np.where(z > 0, z, 0.0))
    np.testing.assert_array_equal(O.act_grad(z, O.RELU), (z > 0).astype(float))


# ---------------------------------------------------------- dispatch / combine
def routed(seed, T, E, k, C, d):
    r = rnd(seed)
    l = r.standard_normal((T, E)).astype(np.float32)
    l[:, 0] += 1.5                                        # expert 0 is over-subscribed
    eidx = O.top_k(l, k)
    keys = r.random(T, dtype=np.float32)
    slot, count, demand, src = O.route(eidx, keys, E, C)
    x = r.standard_normal((T, d))
    return r, l, eidx, slot, count, src, x


@pytest.mark.parametrize("k", [1, 2])
def test_dispatch_rows_are_copies_and_combine_inverts_it(k):
    T, E, C, d = 200, 5, 30 * k, 12
    r, l, eidx, slot, count, src, x = routed(3 + k, T, E, k, C, d)
    Xd = O.dispatch(x, src, k)
    for e in range(E):
        for s in range(C):
            if s < count[e]:
                assert np.array_equal(Xd[e, s], x[src[e, s] // k])
            else:
                assert not Xd[e, s].any()
    back = O.combine_fwd(Xd, eidx, slot, None)
    nkept = (slot >= 0).sum(axis=1)
    assert (nkept == 0).any() and (nkept == k).any()
    np.testing.assert_allclose(back, nkept[:, None] * x, rtol=1e-15)
    assert not back[nkept == 0].any()                     # fully dropped -> exactly zero


def test_combine_weights_and_adjoint_identity():
    T, E, C, d, k = 150, 4, 50, 9, 2
    r, l, eidx, slot, count, src, x = routed(8, T, E, k, C, d)
    g = O.gate_weights(O.softmax(l), eidx)
    Yd = r.standard_normal((E, C, d))
    y = O.combine_fwd(Yd, eidx, slot, g)
    for t in range(0, T, 7):                              # explicit sum, token by token
        want = np.zeros(d)
        for j in range(k):
            if slot[t, j] >= 0:
                want += g[t, j] * Yd[eidx[t, j], slot[t, j]]
        np.testing.assert_allclose(y[t], want, rtol=1e-14, atol=1e-15)
    dy = r.standard_normal((T, d))
    dYd, dg = O.combine_bwd(dy, Yd, eidx, slot, g)
    # <combine(Yd), dy> = <Yd, dYd> on used slots (combine is linear in Yd)
    used = np.zeros((E, C), bool)
    used[eidx[slot >= 0], slot[slot >= 0]] = True
    assert np.vdot(y, dy) == pytest.approx(np.vdot(Yd[used], dYd[used]), rel=1e-12)
    assert not dYd[~used].any()
    # y is linear in g: <y, dy> = sum g * dg
    assert np.vdot(y, dy) == pytest.approx(float((g * dg).sum()), rel=1e-12)
    assert not dg[slot < 0].any()


# ------------------------------------------------------------------ expert FFN
@pytest.mark.parametrize("kind", [O.RELU, O.GELU])
def test_single_expert_layer_is_the_dense_ffn(kind):
    # one expert, capacity >= T: no gate, plain dense FFN (Sec. 5.2's 1-expert model)
    r = rnd(21)
    T, d, f = 6, 5, 7
    x, W1, W2 = r.standard_normal((T, d)), r.standard_normal((1, d, f)), r.standard_normal((1, f, d))
    Wg = r.standard_normal((d, 1))
    out = O.moe_layer(x, Wg, None, W1, W2, None, None, 1, T, kind)
    assert np.array_equal(out["gate_w"], np.ones((T, 1)))
    for t in range(T):
        h = []
        for b in range(f):
            z = math.fsum(x[t, a] * W1[0, a, b] for a in range(d))
            h.append(max(z, 0.0) if kind == O.RELU else 0.5 * z * (1 + math.erf(z / math.sqrt(2))))
        for c in range(d):
            want = math.fsum(h[b] * W2[0, b, c] for b in range(f))
            assert out["y"][t, c] == pytest.approx(want, rel=1e-12, abs=1e-13)


def test_relu_with_positive_preactivations_is_a_product_of_matrices():
    r = rnd(22)
    E, C, d, f = 3, 8, 6, 10
    Xd = r.random((E, C, d)) + 0.1
    W1 = r.random((E, d, f)) + 0.1
    W2 = r.standard_normal((E, f, d))
    count = np.array([8, 3, 0], np.int32)
    Z, H, Yd = O.expert_ffn_fwd(Xd, count, W1, W2, O.RELU)
    for e in range(E):
        n = count[e]
        np.testing.assert_allclose(Yd[e, :n], Xd[e, :n] @ (W1[e] @ W2[e]), rtol=1e-12)
        assert not Yd[e, n:].any() and not Z[e, n:].any()


def test_ffn_bwd_only_counts_kept_rows_and_empty_expert_gets_zero_grads():
    r = rnd(23)
    E, C, d, f = 3, 6, 4, 5
    Xd, dYd = r.standard_normal((E, C, d)), r.standard_normal((E, C, d))
    W1, W2 = r.standard_normal((E, d, f)), r.standard_normal((E, f, d))
    count = np.array([6, 2, 0], np.int32)
    Z, H, Yd = O.expert_ffn_fwd(Xd, count, W1, W2, O.GELU)
    dXd, dW1, dW2 = O.expert_ffn_bwd(dYd, Xd, Z, count, W1, W2, O.GELU)
    assert not dW1[2].any() and not dW2[2].any() and not dXd[2].any()
    # rows beyond the count must not leak into the weight gradients
    Xd2, dYd2 = Xd.copy(), dYd.copy()
    Xd2[1, 2:] = 99.0
    dYd2[1, 2:] = -77.0
    dXd2, dW1b, dW2b = O.expert_ffn_bwd(dYd2, Xd2, Z, count, W1, W2, O.GELU)
    assert np.array_equal(dW1, dW1b) and np.array_equal(dW2, dW2b)
    assert np.array_equal(dXd[1, :2], dXd2[1, :2])


# ------------------------------------------- whole layer: torch autograd, fp64
def torch_layer(x, Wg, bias, W1, W2, eidx, slot, dy, kind):
    """The same layer written separately with torch ops, routing given;
    gradients by autograd."""
    tt = lambda a: torch.tensor(np.asarray(a, np.float64), requires_grad=True)
    x_, Wg_, W1_, W2_ = tt(x), tt(Wg), tt(W1), tt(W2)
    logits = x_ @ Wg_
    if bias is not None:
        logits = logits + torch.tensor(np.asarray(bias, np.float64))
    logits.retain_grad()
    p = torch.softmax(logits, dim=1)
    ei = torch.tensor(eidx.astype(np.int64))
    sel = torch.gather(p, 1, ei)
    g = sel if eidx.shape[1] == 1 else sel / sel.sum(dim=1, keepdim=True)
    g.retain_grad()
    y = torch.zeros_like(x_)
    fn = torch.relu if kind == O.RELU else torch.nn.functional.gelu
    for t in range(x.shape[0]):
        for j in range(eidx.shape[1]):
            if slot[t, j] >= 0:
                e = int(eidx[t, j])
                y = y + torch.nn.functional.one_hot(torch.tensor(t), x.shape[0]).double()[:, None] * (
                    g[t, j] * (fn(x_[t] @ W1_[e]) @ W2_[e]))[None, :]
    (y * torch.tensor(np.asarray(dy, np.float64))).sum().backward()
    z = lambda a: a.grad.numpy() if a.grad is not None else np.zeros(a.shape)
    return dict(y=y.detach().numpy(), dx=z(x_), dWg=z(Wg_), dW1=z(W1_), dW2=z(W2_),
                dlogits=z(logits), dgate_w=z(g))


@pytest.mark.parametrize("k,kind,skew", [(1, O.RELU, False), (2, O.GELU, True), (1, O.GELU, True)])
def test_whole_layer_against_torch_autograd(k, kind, skew):
    r = rnd(30 + k)
    T, d, f, E, C = 40, 8, 12, 4, 9 if k == 1 else 16
    x, dy = r.standard_normal((T, d)), r.standard_normal((T, d))
    Wg = r.standard_normal((d, E)) * 0.5
    W1, W2 = r.standard_normal((E, d, f)) * 0.3, r.standard_normal((E, f, d)) * 0.3
    bias = np.array([1.0, 0, 0, -0.5]) if skew else None
    keys = r.random(T, dtype=np.float32)
    out = O.moe_layer(x, Wg, bias, W1, W2, keys, dy, k, C, kind)
    assert (out["slot"] < 0).any() and (out["slot"] >= 0).any()
    ref = torch_layer(x, Wg, bias, W1, W2, out["expert_idx"], out["slot"], dy, kind)
    for name in ["y", "dx", "dWg", "dW1", "dW2", "dlogits"]:
        np.testing.assert_allclose(out[name], ref[name], rtol=1e-9, atol=1e-12, err_msg=name)
    # autograd's dg includes the (formal) gradient of dropped choices' weights: zero,
    # because dropped choices never enter y
    np.testing.assert_allclose(out["dgate_w"], ref["dgate_w"], rtol=1e-9, atol=1e-12)


def test_fully_dropped_tokens_get_exact_zero_rows():
    for k in (1, 2):
        w = I.small("drop", 96, 8, 16, 3, k, 5)
        d = I.make_inputs(w, seed=k)
        out = O.moe_layer(d["x"], d["Wg"] * 20, None, d["W1"], d["W2"], d["rts_keys"], d["dy"],
                          k, w.capacity, w.act)
        dropped = np.all(out["slot"] < 0, axis=1)
        assert dropped.sum() > 10
        assert not out["y"][dropped].any()
        assert not out["dx_disp"][dropped].any()
        assert not out["dlogits"][dropped].any()
        assert not out["dgate_w"][dropped].any()
        assert not (out["dx"][dropped]).any()


# --------------------------------------------------------- finite differences
def test_backward_against_central_differences():
    w = I.small("fd", 24, 6, 10, 4, 2, 8)
    d = I.make_inputs(w, seed=3)
    x, dy = d["x"].astype(np.float64), d["dy"].astype(np.float64)
    Wg, W1, W2 = d["Wg"].astype(np.float64) * 10, d["W1"].astype(np.float64) * 10, d["W2"].astype(np.float64) * 10
    args = dict(x=x, Wg=Wg, W1=W1, W2=W2)

    def run(a, with_dy=True):
        return O.moe_layer(a["x"], a["Wg"], None, a["W1"], a["W2"], d["rts_keys"],
                           dy if with_dy else None, w.k, w.capacity, w.act)

    base = run(args)
    assert (base["slot"] < 0).any()
    loss = lambda o: float(np.vdot(o["y"], dy))
    r = rnd(4)
    h = 1e-6
    for name, grad in [("x", "dx"), ("Wg", "dWg"), ("W1", "dW1"), ("W2", "dW2")]:
        for _ in range(12):
            idx = tuple(r.integers(0, s) for s in args[name].shape)
            up, dn = dict(args), dict(args)
            up[name] = args[name].copy(); up[name][idx] += h
            dn[name] = args[name].copy(); dn[name][idx] -= h
            ou, od = run(up, False), run(dn, False)
            assert np.array_equal(ou["expert_idx"], base["expert_idx"])     # routing unchanged
            assert np.array_equal(od["slot"], base["slot"])
            fd = (loss(ou) - loss(od)) / (2 * h)
            assert base[grad][idx] == pytest.approx(fd, rel=2e-6, abs=1e-8), (name, idx)


# ----------------------------------------------------------- gate_bwd identities
def test_gate_bwd_identities():
    r = rnd(40)
    T, E = 60, 6
    l = r.standard_normal((T, E)).astype(np.float32)
    p = O.softmax(l)
    e2 = O.top_k(l, 2)
    slot = np.where(r.random((T, 2)) < 0.8, 0, -1).astype(np.int32)
    dg = r.standard_normal((T, 2))
    dl = O.gate_bwd(dg, p, e2, slot)
    np.testing.assert_allclose(dl.sum(axis=1), 0.0, atol=1e-15)       # softmax is shift invariant
    # g0 + g1 = 1: a common shift of (dg0, dg1) changes nothing when both are kept
    both = np.all(slot >= 0, axis=1)
    dl2 = O.gate_bwd(dg + 3.0, p, e2, slot)
    np.testing.assert_allclose(dl2[both], dl[both], atol=1e-14)
    # a dropped choice's dg is ignored
    dg3 = dg.copy()
    dg3[slot < 0] = 123.0
    assert np.array_equal(O.gate_bwd(dg3, p, e2, slot), dl)
    # single expert: probability is the constant 1
    one = O.gate_bwd(r.standard_normal((T, 1)), np.ones((T, 1)), np.zeros((T, 1), np.int32),
                     np.zeros((T, 1), np.int32))
    assert not one.any()
    # k = 1 closed form: dl = dg * p0 * (onehot(e0) - p)
    e1 = O.top_k(l, 1)
    s1 = np.zeros((T, 1), np.int32)
    dg1 = r.standard_normal((T, 1))
    got = O.gate_bwd(dg1, p, e1, s1)
    p0 = p[np.arange(T), e1[:, 0]]
    want = dg1 * p0[:, None] * (np.eye(E)[e1[:, 0]] - p)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-16)


def test_gate_logits_bwd_shapes_and_adjoint():
    r = rnd(41)
    x, Wg, dl = r.standard_normal((9, 5)), r.standard_normal((5, 3)), r.standard_normal((9, 3))
    dWg, dx = O.gate_logits_bwd(x, Wg, dl)
    assert dWg.shape == (5, 3) and dx.shape == (9, 5)
    # <x Wg, dl> is bilinear: its gradient wrt Wg is dWg, wrt x is dx
    assert np.vdot(Wg, dWg) == pytest.approx(np.vdot(x @ Wg, dl), rel=1e-12)
    assert np.vdot(x, dx) == pytest.approx(np.vdot(x @ Wg, dl), rel=1e-12)
