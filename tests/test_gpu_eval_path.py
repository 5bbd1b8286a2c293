"""GPU parity of the forward-only (evaluation) path: capacity factor 2.0
(Sec. 5.1), no saved derivative, and the expert-utilisation count used for
pruning (Sec. 3.3), through the C ABI against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2109_10465_amd import binding as B
from paper_2109_10465_amd import inputs as I
from paper_2109_10465_amd.layer import MoELayer

import gpu_util as G

pytestmark = pytest.mark.gpu


def eval_workload(name, T, d, f, E, k, dtype, act, **kw):
    C = B.moe_capacity(T, E, k, 2.0)
    assert C == O.capacity(T, E, k, 2.0)
    return I.small(name, T, d, f, E, k, C, dtype, act, **kw)


CASES = [
    eval_workload("eval_f32_top1", 900, 72, 264, 7, 1, I.F32, I.GELU, skew="hot0", skew_param=0.5),
    eval_workload("eval_bf16_top2", 1500, 264, 520, 6, 2, I.BF16, I.GELU, skew="zipf", skew_param=1.1),
    eval_workload("eval_bf16_relu", 2049, 128, 136, 9, 1, I.BF16, I.RELU, skew="hot0", skew_param=0.6),
]


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_forward_only_matches_the_oracle_over_several_batches(w):
    layer = MoELayer(w.T, w.d_model, w.d_ff, w.E, w.k, w.capacity, w.dtype, w.act, forward_only=True)
    assert layer.dact is None and not hasattr(layer, "dW1")
    batches = []
    for seed in (21, 22, 23):
        d = I.make_inputs(w, seed=seed)
        d["Wg"] = d["Wg"] * 8.0
        _, lg32 = G.oracle_logits(d)
        ref = O.moe_layer(d["x"], d["Wg"], d["bias"], d["W1"], d["W2"], d["rts_keys"], None, w.k, w.capacity,
                          w.act, logits=lg32)
        print(f"[gpu] {w.name} seed {seed} forward-only", flush=True)
        layer.forward(G.to_dev(d["x"], w.dtype), G.to_dev(d["Wg"], I.F32), G.to_dev(d["bias"], I.F32),
                      G.to_dev(d["W1"], w.dtype), G.to_dev(d["W2"], w.dtype), G.to_dev(d["rts_keys"], I.F32),
                      logits=G.to_dev(lg32, I.F32))
        torch.cuda.synchronize()
        for n in G.INT_NAMES:
            assert np.array_equal(G.host(getattr(layer, n)), ref[n]), n
        m = G.row_mask(ref["expert_count"], w.capacity)
        tol = G.TOL[w.dtype]
        assert G.rel_l2(G.host(layer.h)[m], ref["H"][m]) <= tol
        assert G.rel_l2(G.host(layer.yd)[m], ref["Yd"][m]) <= tol
        assert G.rel_l2(G.host(layer.y), ref["y"]) <= tol
        batches.append(ref["expert_idx"])
        # running utilisation after this batch
        assert np.array_equal(G.host(layer.utilisation), O.utilisation(batches, w.E))
    with pytest.raises(B.MoeError):
        layer.backward(None)


def test_forward_only_h_equals_the_training_forward_bit_for_bit():
    """Dropping the derivative changes nothing else: h, yd and y of the forward-only
    call equal those of the training forward exactly."""
    w = CASES[1]
    d = I.make_inputs(w, seed=5)
    a = MoELayer(w.T, w.d_model, w.d_ff, w.E, w.k, w.capacity, w.dtype, w.act)
    b = MoELayer(w.T, w.d_model, w.d_ff, w.E, w.k, w.capacity, w.dtype, w.act, forward_only=True)
    args = (G.to_dev(d["x"], w.dtype), G.to_dev(d["Wg"], I.F32), G.to_dev(d["bias"], I.F32),
            G.to_dev(d["W1"], w.dtype), G.to_dev(d["W2"], w.dtype), G.to_dev(d["rts_keys"], I.F32))
    a.forward(*args); b.forward(*args)
    torch.cuda.synchronize()
    m = torch.from_numpy(G.row_mask(G.host(a.expert_count), w.capacity)).cuda()
    for n in ("h", "yd"):
        assert torch.equal(getattr(a, n)[m], getattr(b, n)[m]), n
    assert torch.equal(a.y, b.y)
