"""Pins of the oracle's seeded noise: the Philox4x32-10 generator against its
published known-answer vectors, the gate jitter (Sec. 5.1) and the expert
dropout (Sec. 5.4) against their definitions, statistics, torch autograd and the
noise-free special cases."""
import os

import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2109_10465_amd import inputs as I

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_known_answers.txt")


def test_philox_known_answers():
    n = 0
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(v, 16) for v in line.split()]
        out = O.philox4x32(*w[:6])
        assert [int(v) for v in out] == w[6:]
        n += 1
    assert n == 3


def test_word_layout_and_streams():
    w = O.random_words(10, seed=(7 << 32) | 5, stream=O.STREAM_JITTER)
    # element i = word i % 4 of the block with counter (i // 4, 0, stream, 0), key (seed lo, seed hi)
    for i in (0, 3, 4, 9):
        blk = O.philox4x32(i // 4, 0, O.STREAM_JITTER, 0, 5, 7)
        assert int(w[i]) == int(blk[i % 4])
    assert not np.array_equal(w, O.random_words(10, (7 << 32) | 5, O.STREAM_DROPOUT))
    assert not np.array_equal(w, O.random_words(10, (7 << 32) | 6, O.STREAM_JITTER))
    assert np.array_equal(w[:6], O.random_words(6, (7 << 32) | 5, O.STREAM_JITTER))     # prefix-stable


def test_jitter_noise_is_uniform_in_its_band():
    eps = 0.01
    nz = O.jitter_noise(400, 256, eps, seed=3)
    assert nz.shape == (400, 256) and nz.min() >= 1 - eps and nz.max() < 1 + eps
    u = (nz - (1 - eps)) / (2 * eps)
    assert abs(u.mean() - 0.5) < 4 / np.sqrt(12 * u.size)
    hist = np.histogram(u, bins=16, range=(0, 1))[0]
    chi2 = ((hist - u.size / 16) ** 2 / (u.size / 16)).sum()
    assert chi2 < 45                                   # 15 dof: p ~ 1e-4
    assert np.array_equal(O.jitter_noise(400, 256, 0.0, 3), np.ones((400, 256)))


def test_dropout_scale_keep_rate_and_values():
    p = 0.4
    sc = O.dropout_scale(4, 100, 64, p, seed=9)
    assert set(np.unique(sc)) == {0.0, 1.0 / (1 - p)}
    n = sc.size
    assert abs((sc > 0).mean() - (1 - p)) < 4 * np.sqrt(p * (1 - p) / n)
    assert abs(sc.mean() - 1.0) < 4 * np.sqrt(p / (1 - p) / n)          # inverted dropout keeps the mean
    # the threshold is floor(p 2^32) on the element's word
    w = O.random_words(n, 9, O.STREAM_DROPOUT).reshape(sc.shape)
    assert np.array_equal(sc > 0, w >= int(np.floor(p * 2.0 ** 32)))


def test_layer_with_noise_matches_torch_autograd_and_reduces_to_plain():
    w = I.small("noise", 200, 16, 24, 4, 2, 120, I.F32, I.GELU)
    d = I.make_inputs(w, seed=6)
    d["Wg"] = d["Wg"] * 10
    plain = O.moe_layer(d["x"], d["Wg"], d["bias"], d["W1"], d["W2"], d["rts_keys"], d["dy"], w.k, w.capacity, w.act)
    same = O.moe_layer(d["x"], d["Wg"], d["bias"], d["W1"], d["W2"], d["rts_keys"], d["dy"], w.k, w.capacity, w.act,
                       jitter_eps=0.0, drop_p=0.0, seed=77)
    for n in ("y", "dx", "dW1", "dWg"):
        assert np.array_equal(plain[n], same[n])
    eps, p, seed = 0.05, 0.4, 1234
    out = O.moe_layer(d["x"], d["Wg"], d["bias"], d["W1"], d["W2"], d["rts_keys"], d["dy"], w.k, w.capacity, w.act,
                      jitter_eps=eps, drop_p=p, seed=seed)
    assert not np.array_equal(out["logits"], plain["logits"]) and not np.array_equal(out["y"], plain["y"])
    # independent forward in torch (fp64) with the oracle's routing and noise as constants
    nz = torch.tensor(O.jitter_noise(w.T, w.d_model, eps, seed))
    sc = torch.tensor(O.dropout_scale(w.E, w.capacity, w.d_ff, p, seed))
    x = torch.tensor(d["x"], dtype=torch.float64, requires_grad=True)
    Wg = torch.tensor(d["Wg"], dtype=torch.float64, requires_grad=True)
    W1 = torch.tensor(d["W1"], dtype=torch.float64, requires_grad=True)
    W2 = torch.tensor(d["W2"], dtype=torch.float64, requires_grad=True)
    logits = (x * nz) @ Wg
    if d["bias"] is not None:
        logits = logits + torch.tensor(d["bias"], dtype=torch.float64)
    assert np.allclose(logits.detach().numpy(), out["logits"], atol=1e-12)
    probs = torch.softmax(logits, dim=1)
    eidx, slot = out["expert_idx"], out["slot"]
    y = torch.zeros_like(x)
    for t in range(w.T):
        pe = probs[t, eidx[t].astype(np.int64)]
        gw = pe / pe.sum()
        for j in range(w.k):
            if slot[t, j] < 0:
                continue
            e, s = int(eidx[t, j]), int(slot[t, j])
            h = torch.nn.functional.gelu(x[t] @ W1[e]) * sc[e, s]      # the experts see x, not x * noise
            y[t] = y[t] + gw[j] * (h @ W2[e])
    assert np.allclose(y.detach().numpy(), out["y"], atol=1e-12)
    (y * torch.tensor(d["dy"], dtype=torch.float64)).sum().backward()
    for name, t_ in (("dx", x), ("dWg", Wg), ("dW1", W1), ("dW2", W2)):
        assert np.allclose(t_.grad.numpy(), out[name], atol=1e-11), name
