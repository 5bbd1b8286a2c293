"""The sampled-output checker used on full-size GPU runs is itself checked on
the CPU: fed the oracle's own full result it passes; with a planted mistake in
any sampled quantity it fails."""
import numpy as np
import pytest

from oracle import moe_oracle as O
from paper_2109_10465_amd import inputs as I

import gpu_util as G


def full_result(w, d):
    lg = O.gate_logits(d["x"], d["Wg"], d["bias"]).astype(np.float32)
    out = O.moe_layer(d["x"], d["Wg"], d["bias"], d["W1"], d["W2"], d["rts_keys"], d["dy"], w.k,
                      w.capacity, w.act, logits=lg)
    got = {k.lower() if k in ("Xd", "Z", "H", "Yd") else {"dYd": "dyd", "dXd": "dxd"}.get(k, k): v
           for k, v in out.items()}
    got["logits"] = lg
    got["dact"] = O.act_grad(out["Z"], w.act)
    return got


@pytest.mark.parametrize("k", [1, 2])
def test_sampled_checker_accepts_the_oracle_and_rejects_planted_errors(k):
    w = I.small("harness", 400, 16, 40, 5, k, 60 * k, I.F32, I.GELU, skew="hot0", skew_param=0.5)
    d = I.make_inputs(w, seed=2)
    d["Wg"] = d["Wg"] * 10
    got = full_result(w, d)
    fetch = lambda name, e: got[name][e]
    G.check_sampled(w, d, got, n_tokens=60, n_cols=8, n_rows=10, fetch_expert=fetch)
    for name in ["y", "dx", "dgate_w", "dlogits", "dW1", "dW2", "yd", "dxd", "dWg", "dact"]:
        bad = dict(got)
        bad[name] = got[name] * 1.001 + 1e-3
        with pytest.raises(AssertionError):
            G.check_sampled(w, d, bad, n_tokens=60, n_cols=8, n_rows=10,
                            fetch_expert=lambda n, e: bad[n][e])
    bad = dict(got)
    bad["slot"] = got["slot"].copy()
    bad["slot"][0, 0] ^= 1
    with pytest.raises(AssertionError):
        G.check_sampled(w, d, bad, n_tokens=60, n_cols=8, n_rows=10, fetch_expert=fetch)


def test_row_bound_rejects_one_wrong_row_that_the_tensor_norm_lets_through():
    """bf16 bar (2e-2 over the whole tensor): one entirely wrong row of a few thousand changes the norm by about a
    per cent and would pass; the per-row bound must reject it, and so must the full comparison of a bf16 layer."""
    rng = np.random.default_rng(0)
    want = rng.standard_normal((16384, 64))
    got = want * (1.0 + 2e-3 * rng.standard_normal(want.shape))          # bf16-like rounding noise
    G.assert_rows("clean", got, want, 2e-2)
    bad = got.copy()
    bad[1234] = rng.standard_normal(64)                                   # a row of something else
    assert G.rel_l2(bad, want) < 2e-2                                     # the tensor-wide bound does not see it
    with pytest.raises(AssertionError):
        G.assert_rows("planted", bad, want, 2e-2)
    spike = got.copy()
    spike[7, 3] += 0.5 * np.abs(want).max()                               # one wild element
    with pytest.raises(AssertionError):
        G.assert_rows("spike", spike, want, 2e-2)
    # the same through the comparison the GPU tests use, on a bf16 layer
    w = I.small("rowbound", 2048, 16, 24, 4, 2, 1100, I.BF16, I.GELU)
    d = I.make_inputs(w, seed=5)
    res = full_result(w, d)
    lg = res["logits"]
    ref = O.moe_layer(d["x"], d["Wg"], d["bias"], d["W1"], d["W2"], d["rts_keys"], d["dy"], w.k, w.capacity, w.act,
                      logits=lg)
    G.compare_full(w, d, res, ref)
    for name in ["y", "dx"]:
        bad = dict(res)
        bad[name] = res[name].copy()
        t = int(np.nonzero((ref["slot"] >= 0).all(axis=1))[0][3])
        bad[name][t] = bad[name][t] * 1.5
        assert G.rel_l2(bad[name], ref[name]) < 2e-2
        with pytest.raises(AssertionError):
            G.compare_full(w, d, bad, ref)


def test_chained_routing_checker_near_ties_and_planted_errors():
    """The checker of the chained path accepts a run whose logits differ in the
    last bits, accepts either order of a near-tied pair (with the slots that
    follow from it), and rejects a wrong choice on a clear-cut token."""
    w = I.small("chain", 300, 16, 24, 6, 2, 70, I.F32, I.GELU)
    d = I.make_inputs(w, seed=4)
    d["Wg"] = d["Wg"] * 10
    lg = O.gate_logits(d["x"], d["Wg"], d["bias"]).astype(np.float32)
    # plant a near tie: token 5's best two logits differ by one fp32 ulp
    e = O.top_k(lg, 2)
    lg[5, e[5, 1]] = np.nextafter(lg[5, e[5, 0]], np.float32(-np.inf))
    route_of = lambda eidx: dict(zip(["slot", "expert_count", "expert_demand", "slot_src"],
                                     O.route(eidx, d["rts_keys"], w.E, w.capacity)), expert_idx=eidx)
    eidx = O.top_k(lg, 2)
    ref = route_of(eidx)
    noisy = (lg.astype(np.float64) * (1 + 2e-7 * np.sin(np.arange(lg.size)).reshape(lg.shape))).astype(np.float32)
    got = dict(ref, logits=noisy)
    assert G.check_chained_routing(w, d, got, lg, ref) >= 1
    flipped = eidx.copy()
    flipped[5] = flipped[5, ::-1]                       # the other order of the near-tied pair
    assert G.check_chained_routing(w, d, dict(route_of(flipped), logits=noisy), lg, ref) >= 1
    with pytest.raises(AssertionError):                  # right choice, stale slots
        G.check_chained_routing(w, d, dict(ref, expert_idx=flipped, logits=noisy), lg, ref)
    wrong = eidx.copy()
    t = int(np.argmax(np.sort(lg, axis=1)[:, -1] - np.sort(lg, axis=1)[:, -2]))   # clearest winner
    wrong[t] = wrong[t, ::-1]
    with pytest.raises(AssertionError):
        G.check_chained_routing(w, d, dict(route_of(wrong), logits=noisy), lg, ref)
    assert G.check_chained_routing(w, d, dict(ref, logits=lg), lg, ref) >= 0
