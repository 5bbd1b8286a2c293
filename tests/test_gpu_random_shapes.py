"""GPU parity on a seeded sweep of random small shapes and option mixes: every
output of the HIP layer (through the C ABI) against the CPU oracle, routed on
the oracle's fp32 logits.  Shapes cover ragged sizes in every dimension, 1..256
experts, both dtypes and activations, top-1/top-2, RTS and position priority,
and random mixes of the balancing loss, grouped selection, jitter and dropout."""
import numpy as np
import pytest

from oracle import moe_oracle as O
from paper_2109_10465_amd import inputs as I

import gpu_util as G

pytestmark = pytest.mark.gpu


def make_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        k = int(rng.integers(1, 3))
        E = int(rng.choice([1, 2, 3, 4, 5, 8, 13, 32, 33, 64, 100, 128, 255, 256]))
        E = max(E, k)
        dtype = int(rng.integers(0, 2))
        act = int(rng.integers(0, 2))
        d = 8 * int(rng.integers(1, 40))
        f = 8 * int(rng.integers(1, 60))
        groups = int(rng.choice([1, 1, 1, 2, 4]))
        if groups > 1:
            T = 256 * groups * int(rng.integers(1, 3))
        else:
            T = int(rng.integers(1, 3000))
        cf = float(rng.choice([0.5, 1.0, 1.25, 2.0]))
        C = max(1, int(np.ceil(k * cf * T / E)))
        if groups > 1:
            C = max(groups, (C // groups) * groups)
        if E * C * max(d, f) > 3.0e7:          # keep the oracle quick
            f = max(8, f // 4 // 8 * 8)
            d = max(8, d // 2 // 8 * 8)
        skew = rng.choice(["none", "hot0", "zipf"]) if E >= 4 else "none"
        w = I.small(f"rnd{i}", T, d, f, E, k, C, dtype, act, skew=str(skew),
                    skew_param=0.4 if skew == "hot0" else 1.1)
        opts = dict(use_keys=bool(rng.integers(0, 2)), aux_coef=float(rng.choice([0.0, 0.01])), groups=groups,
                    jitter_eps=float(rng.choice([0.0, 0.02])), drop_p=float(rng.choice([0.0, 0.3])))
        cases.append((w, opts))
    return cases


CASES = make_cases(40, seed=2024)


@pytest.mark.parametrize("w,opts", CASES, ids=lambda v: v.name if hasattr(v, "name") else "")
def test_random_shape(w, opts):
    seed = 99
    d = I.make_inputs(w, seed=31)
    d["Wg"] = d["Wg"] * 6.0
    keys = d["rts_keys"] if opts["use_keys"] else None
    _, lg32 = G.oracle_logits(d, opts["jitter_eps"], seed)
    ref = O.moe_layer(d["x"], d["Wg"], d["bias"], d["W1"], d["W2"], keys, d["dy"], w.k, w.capacity, w.act,
                      logits=lg32, aux_coef=opts["aux_coef"], groups=opts["groups"],
                      jitter_eps=opts["jitter_eps"], drop_p=opts["drop_p"], seed=seed)
    print(w.name, f"T={w.T} d={w.d_model} f={w.d_ff} E={w.E} k={w.k} C={w.capacity} dtype={w.dtype} act={w.act}", opts,
          flush=True)
    _, got = G.run_layer(w, d, opts["use_keys"], logits=lg32, aux_coef=opts["aux_coef"], groups=opts["groups"],
                         jitter_eps=opts["jitter_eps"], drop_p=opts["drop_p"], seed=seed)
    sc = O.dropout_scale(w.E, w.capacity, w.d_ff, opts["drop_p"], seed) if opts["drop_p"] > 0 else None
    G.compare_full(w, d, got, ref, aux=opts["aux_coef"] != 0.0, scale=sc)
    if opts["aux_coef"] != 0.0:
        assert abs(float(got["aux_loss"][0]) - ref["aux_loss"]) <= 1e-5 * ref["aux_loss"]
