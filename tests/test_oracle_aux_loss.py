"""Pins of the oracle's balancing loss (Sec. 5.1, "MoE setting") against a
hand-worked case, closed forms, torch autograd in fp64 and finite differences."""
import os

import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2109_10465_amd import inputs as I

GOLD = os.path.join(os.path.dirname(__file__), "golden", "aux_loss_worked_case.txt")


def read_gold():
    out = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        out[k] = np.array([float(a) for a in v])
    return out


def test_hand_worked_case():
    g = read_gold()
    p = g["probs"].reshape(4, 2)
    eidx = g["first"].astype(np.int32).reshape(4, 1)
    assert np.array_equal(O.top_k(np.log(np.maximum(p, 1e-300)), 1), eidx)   # ties -> smaller id
    L, f, P = O.aux_loss(p, eidx)
    assert np.allclose(f, g["f"], atol=0) and np.allclose(P, g["P"], atol=1e-15)
    assert abs(L - g["L"][0]) < 1e-15
    dl = O.aux_loss_bwd(p, f, 1.0)
    assert np.allclose(dl.ravel(), g["dl"], atol=1e-15)


@pytest.mark.parametrize("E", [2, 5, 32])
def test_uniform_gate_gives_one_and_collapse_gives_E(E):
    T = 6 * E
    p = np.full((T, E), 1.0 / E)
    eidx = (np.arange(T) % E).astype(np.int32)[:, None]         # perfectly balanced first choices
    L, f, P = O.aux_loss(p, eidx)
    assert abs(L - 1.0) < 1e-14 and np.allclose(f, 1.0 / E) and np.allclose(P, 1.0 / E)
    assert np.abs(O.aux_loss_bwd(p, f, 0.01)).max() < 1e-17      # uniform dp: softmax kills it
    # every token sure of expert 2 % E: f and P are one-hot, L = E
    q = np.zeros((T, E)); q[:, 2 % E] = 1.0
    L2, _, _ = O.aux_loss(q, np.full((T, 1), 2 % E, np.int32))
    assert abs(L2 - E) < 1e-14


def test_only_first_choices_count_for_top2():
    rng = np.random.default_rng(0)
    lg = rng.standard_normal((200, 6))
    p = O.softmax(lg)
    e2 = O.top_k(lg, 2)
    L2, f2, _ = O.aux_loss(p, e2)
    L1, f1, _ = O.aux_loss(p, e2[:, :1])
    assert L1 == L2 and np.array_equal(f1, f2)
    assert np.array_equal(f2 * 200, np.bincount(np.argmax(lg, axis=1), minlength=6))
    assert abs(f2.sum() - 1.0) < 1e-15


def test_gradient_matches_torch_autograd_and_finite_differences():
    rng = np.random.default_rng(1)
    T, E, coef = 37, 7, 0.01
    lg = rng.standard_normal((T, E)) * 2
    p = O.softmax(lg)
    eidx = O.top_k(lg, 1)
    L, f, P = O.aux_loss(p, eidx)
    dl = O.aux_loss_bwd(p, f, coef)
    # torch: the same objective written with library ops, f detached by construction
    tl = torch.tensor(lg, dtype=torch.float64, requires_grad=True)
    tp = torch.softmax(tl, dim=1)
    tf = torch.bincount(torch.argmax(tl, dim=1), minlength=E).double() / T
    tL = E * (tf * tp.mean(dim=0)).sum()
    assert abs(float(tL.detach()) - L) < 1e-14
    (coef * tL).backward()
    assert np.allclose(dl, tl.grad.numpy(), atol=1e-16, rtol=1e-12)
    # central differences on a few entries (the first choices do not change for eps this small)
    eps = 1e-6
    for (t, e) in [(0, 0), (5, 3), (36, 6), (17, 2)]:
        up, dn = lg.copy(), lg.copy()
        up[t, e] += eps; dn[t, e] -= eps
        Lu = E * np.dot(f, O.softmax(up).mean(axis=0))
        Ld = E * np.dot(f, O.softmax(dn).mean(axis=0))
        assert abs(coef * (Lu - Ld) / (2 * eps) - dl[t, e]) < 1e-10
    assert np.abs(dl.sum(axis=1)).max() < 1e-17                  # softmax gradients sum to zero per token


def test_layer_adds_the_term_for_every_token_dropped_or_not():
    w = I.small("aux", 300, 16, 24, 6, 2, 40, I.F32, I.GELU, skew="hot0", skew_param=0.5)
    d = I.make_inputs(w, seed=3)
    a = O.moe_layer(d["x"], d["Wg"], d["bias"], d["W1"], d["W2"], d["rts_keys"], d["dy"], w.k, w.capacity, w.act)
    b = O.moe_layer(d["x"], d["Wg"], d["bias"], d["W1"], d["W2"], d["rts_keys"], d["dy"], w.k, w.capacity, w.act,
                    aux_coef=0.01)
    extra = b["dlogits"] - a["dlogits"]
    assert np.allclose(extra, O.aux_loss_bwd(a["probs"], a["first_frac"], 0.01), atol=1e-18)
    dropped = np.all(a["slot"] < 0, axis=1)
    assert dropped.any() and np.abs(extra[dropped]).max() > 0    # dropped tokens still feel the balancing loss
    assert a["aux_loss"] == b["aux_loss"] and a["aux_loss"] > 1.0    # a skewed gate is above the uniform value
    for n in ("y", "dW1", "dW2"):
        assert np.array_equal(a[n], b[n])
    assert not np.array_equal(a["dWg"], b["dWg"]) and not np.array_equal(a["dx"], b["dx"])
