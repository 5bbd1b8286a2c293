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
