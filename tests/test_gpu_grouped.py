"""GPU parity of grouped token selection (Sec. 3.1 group dimension; the second
arm of the Sec. 5.5 ablation) through the C ABI against the CPU oracle: routing
bit-exact, every float output within tolerance."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2109_10465_amd import binding as B
from paper_2109_10465_amd import inputs as I

import gpu_util as G

pytestmark = pytest.mark.gpu

CASES = [
    # (workload, groups): group size a multiple of 256 tokens, capacity a multiple of the group count
    (I.small("grp_f32_top1", 1024, 72, 136, 7, 1, 160, I.F32, I.GELU, skew="hot0", skew_param=0.5), 4),
    (I.small("grp_bf16_top2", 2048, 136, 264, 6, 2, 704, I.BF16, I.GELU, skew="zipf", skew_param=1.1), 8),
    (I.small("grp_many_experts", 4096, 64, 64, 200, 2, 48, I.BF16, I.RELU, skew="zipf", skew_param=1.1), 2),
    (I.small("grp_capacity_one_per_group", 1536, 16, 32, 8, 2, 6, I.F32, I.RELU), 6),
    (I.small("grp_single_group", 777, 40, 72, 5, 2, 200, I.F32, I.GELU, skew="hot0", skew_param=0.5), 1),
]


@pytest.mark.parametrize("w,groups", CASES, ids=lambda v: v.name if hasattr(v, "name") else f"G{v}")
@pytest.mark.parametrize("use_keys", [True, False], ids=["rts", "position"])
def test_grouped_selection_full(w, groups, use_keys):
    d = I.make_inputs(w, seed=17)
    d["Wg"] = d["Wg"] * 8.0
    keys = d["rts_keys"] if use_keys else None
    _, lg32 = G.oracle_logits(d)
    ref = O.moe_layer(d["x"], d["Wg"], d["bias"], d["W1"], d["W2"], keys, d["dy"], w.k, w.capacity, w.act,
                      logits=lg32, groups=groups)
    _, got = G.run_layer(w, d, use_keys, logits=lg32, groups=groups)
    errs = G.compare_full(w, d, got, ref)
    print(w.name, groups, {k: f"{v:.1e}" for k, v in errs.items() if k in ("y", "dx", "dW1")})
    if groups > 1:
        plain = O.route(ref["expert_idx"], keys, w.E, w.capacity)[0]
        assert not np.array_equal(plain, ref["slot"])      # grouping really changes who is kept where


def test_grouped_full_size_cfg3_routing():
    """cfg3 at full size with 8 groups of 2048 tokens: the routing integers in
    full against the oracle (the float path downstream is the plain one)."""
    w = I.WORKLOADS["cfg3"]
    d = I.make_inputs(w, seed=0, with_weights=False)
    _, lg32 = G.oracle_logits(d)
    eidx = O.top_k(lg32, w.k)
    slot, count, demand, slot_src = O.route_grouped(eidx, d["rts_keys"], w.E, w.capacity, 8)
    shape = B.make_shape(w.T, w.d_model, w.d_ff, w.E, w.k, w.capacity, w.dtype, w.act)
    ws = torch.empty(B.moe_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    i32, f32 = torch.int32, torch.float32
    mk = lambda shp, dt: torch.empty(shp, dtype=dt, device="cuda")
    probs, ei, gw, sl = mk((w.T, w.E), f32), mk((w.T, w.k), i32), mk((w.T, w.k), f32), mk((w.T, w.k), i32)
    cnt, dem, src = mk((w.E,), i32), mk((w.E,), i32), mk((w.E, w.capacity), i32)
    B.moe_gate_route_grouped(shape, 8, G.to_dev(lg32, I.F32), G.to_dev(d["rts_keys"], I.F32), probs, ei, gw, sl,
                             cnt, dem, src, ws)
    torch.cuda.synchronize()
    for got, want, n in ((ei, eidx, "expert_idx"), (sl, slot, "slot"), (cnt, count, "expert_count"),
                         (dem, demand, "expert_demand"), (src, slot_src, "slot_src")):
        assert np.array_equal(G.host(got), want), n


def test_grouped_argument_errors():
    shape = B.make_shape(1024, 16, 16, 4, 1, 64, B.F32, 0)
    ws = torch.empty(B.moe_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    t = lambda shp, dt=torch.float32: torch.zeros(shp, dtype=dt, device="cuda")
    args = (t((1024, 4)), None, t((1024, 4)), t((1024, 1), torch.int32), t((1024, 1)), t((1024, 1), torch.int32),
            t((4,), torch.int32), t((4,), torch.int32), t((4, 64), torch.int32), ws)
    for bad in (0, 3, 8, 5):      # 3, 5: T % G; 8: group of 128 tokens; 0: no groups
        with pytest.raises(B.MoeError):
            B.moe_gate_route_grouped(shape, bad, *args)
    B.moe_gate_route_grouped(shape, 4, *args)
    B.moe_gate_route_grouped(shape, 2, *args)
    shape2 = B.make_shape(1024, 16, 16, 4, 1, 66, B.F32, 0)     # capacity not a multiple of 4
    with pytest.raises(B.MoeError):
        B.moe_gate_route_grouped(shape2, 4, *args[:8], t((4, 66), torch.int32), ws)


def test_grouped_selection_with_long_segments():
    """Groups whose (expert, choice) segments hold thousands of candidates: the bucketed ranking path with
    per-group segment tables and per-group row offsets, routing integers in full against the oracle."""
    rng = np.random.default_rng(23)
    T, E, k, groups, C = 16384, 3, 2, 2, 4096
    logits = rng.standard_normal((T, E)).astype(np.float32)
    keys = (np.floor(rng.random(T) * 64) / 64).astype(np.float32)          # many equal keys
    eidx = O.top_k(logits, k)
    slot, count, demand, slot_src = O.route_grouped(eidx, keys, E, C, groups)
    assert demand.max() // groups > 4 * 256 and (slot < 0).any()
    shape = B.make_shape(T, 64, 128, E, k, C, I.F32, I.RELU)
    ws = torch.empty(B.moe_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    i32, f32 = torch.int32, torch.float32
    mk = lambda shp, dt: torch.empty(shp, dtype=dt, device="cuda")
    probs, ei, gw, sl = mk((T, E), f32), mk((T, k), i32), mk((T, k), f32), mk((T, k), i32)
    cnt, dem, src = mk((E,), i32), mk((E,), i32), mk((E, C), i32)
    print("[gpu] grouped routing, long segments", flush=True)
    B.moe_gate_route_grouped(shape, groups, G.to_dev(logits, I.F32), G.to_dev(keys, I.F32), probs, ei, gw, sl,
                             cnt, dem, src, ws)
    torch.cuda.synchronize()
    for got, want, n in ((ei, eidx, "expert_idx"), (sl, slot, "slot"), (cnt, count, "expert_count"),
                         (dem, demand, "expert_demand"), (src, slot_src, "slot_src")):
        assert np.array_equal(G.host(got), want), n
