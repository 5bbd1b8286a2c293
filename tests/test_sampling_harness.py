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
