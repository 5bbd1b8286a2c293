"""GPU parity: the HIP MoE layer (through the C ABI) against the CPU oracle,
element by element, on seeded inputs that span several tiles and ragged tails,
plus the edge cases of the method.  Integers bit-exact; floats within rel-L2
1e-5 (fp32) / 2e-2 (bf16)."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2109_10465_amd import binding as B
from paper_2109_10465_amd import inputs as I

import gpu_util as G

pytestmark = pytest.mark.gpu


def test_library_is_loaded_and_gpu_is_gfx950():
    assert torch.cuda.is_available()
    B.lib()
    assert "gfx950" in torch.cuda.get_device_properties(0).gcnArchName


@pytest.mark.parametrize("name", ["cfg1", "cfg2"])
def test_fp32_workloads_full(name):
    w = I.WORKLOADS[name]
    d = I.make_inputs(w, seed=0)
    _, got = G.run_layer(w, d)
    ref, errs = G.check_full(w, d, got)
    print(name, {k: f"{v:.2e}" for k, v in errs.items()})
    if name == "cfg2":      # skewed gate: the hot expert overflows
        assert ref["expert_demand"][0] > w.capacity and (ref["slot"] < 0).any()


RAGGED = [
    # several tiles in every dimension plus ragged tails; E not a power of two
    I.small("rag_f32_top2", 777, 136, 328, 5, 2, 200, I.F32, I.GELU, skew="hot0", skew_param=0.5),
    I.small("rag_f32_top1", 1000, 72, 264, 7, 1, 130, I.F32, I.RELU, skew="hot0", skew_param=0.4),
    I.small("rag_bf16_top2", 1500, 264, 520, 6, 2, 400, I.BF16, I.GELU, skew="hot0", skew_param=0.45),
    I.small("rag_bf16_top1", 2049, 320, 136, 9, 1, 300, I.BF16, I.GELU, skew="zipf", skew_param=1.1),
    I.small("many_experts", 4096, 64, 64, 200, 2, 48, I.BF16, I.RELU, skew="zipf", skew_param=1.1),
    I.small("relu_bf16", 512, 128, 256, 4, 2, 256, I.BF16, I.RELU),
]


@pytest.mark.parametrize("w", RAGGED, ids=lambda w: w.name)
@pytest.mark.parametrize("use_keys", [True, False], ids=["rts", "position"])
def test_ragged_shapes_full(w, use_keys):
    d = I.make_inputs(w, seed=7)
    d["Wg"] = d["Wg"] * 8.0         # sharper gate -> wider spread of probabilities
    _, got = G.run_layer(w, d, use_keys)
    ref, errs = G.check_full(w, d, got, use_keys)
    print(w.name, {k: f"{v:.2e}" for k, v in errs.items()})


EDGE = [
    I.small("one_token", 1, 8, 8, 2, 1, 1),
    I.small("three_tokens_top2", 3, 16, 24, 2, 2, 2),
    I.small("E_equals_k", 200, 32, 64, 2, 2, 150),
    I.small("single_expert", 300, 32, 64, 1, 1, 300),          # plain dense FFN, no gate
    I.small("capacity_one", 500, 16, 32, 8, 2, 1),
    I.small("nothing_dropped", 256, 24, 40, 4, 2, 600),
    I.small("min_dims_bf16", 130, 8, 8, 3, 1, 50, I.BF16),
]


@pytest.mark.parametrize("w", EDGE, ids=lambda w: w.name)
def test_edge_cases(w):
    d = I.make_inputs(w, seed=11)
    d["Wg"] = d["Wg"] * 10.0
    _, got = G.run_layer(w, d)
    ref, _ = G.check_full(w, d, got)
    if w.name == "single_expert":
        assert np.all(got["gate_w"] == 1.0) and not got["dlogits"].any()
    if w.name == "nothing_dropped":
        assert np.all(ref["slot"] >= 0)


def test_all_tokens_choose_one_expert_and_empty_experts():
    # a huge bias sends every first choice to expert 3; experts 5..7 get a
    # large negative bias and stay empty: zero weight gradients, unused slots -1
    w = I.small("hot_and_empty", 900, 64, 128, 8, 2, 300, I.BF16)
    d = I.make_inputs(w, seed=5)
    bias = np.zeros(8, np.float32)
    bias[3] = 50.0
    bias[5:] = -50.0
    d["bias"] = bias
    _, got = G.run_layer(w, d)
    ref, _ = G.check_full(w, d, got)
    assert ref["expert_demand"][3] == 900 and ref["expert_count"][3] == 300
    assert not ref["expert_count"][5:].any()
    assert not got["dW1"][5:].any() and not got["dW2"][5:].any()
    assert np.all(got["slot_src"][5:] == -1)


def test_duplicate_keys_fall_back_to_token_order():
    w = I.small("dup_keys", 3000, 32, 32, 4, 2, 700)
    d = I.make_inputs(w, seed=13)
    d["rts_keys"] = (np.floor(d["rts_keys"] * 5) / 5).astype(np.float32)   # 5 distinct keys
    _, got = G.run_layer(w, d)
    G.check_full(w, d, got)


def test_combine_of_dispatch_with_unit_weights_is_identity_on_kept_tokens():
    w = I.small("identity", 1200, 96, 64, 6, 2, 150, I.BF16, skew="hot0", skew_param=0.6)
    d = I.make_inputs(w, seed=17)
    d["Wg"] = d["Wg"] * 8.0
    d["bias"] = d["bias"] * 8.0
    layer, got = G.run_layer(w, d)
    x = G.to_dev(d["x"], w.dtype)
    back = torch.empty_like(x)
    B.moe_combine_fwd(layer.shape, layer.xd, layer.expert_idx, layer.slot, None, back)
    torch.cuda.synchronize()
    nkept = (got["slot"] >= 0).sum(axis=1)
    back = G.host(back)
    assert (nkept == 0).any() and (nkept == 2).any()
    # bf16: x and 2x are exact, so the identity holds bit for bit
    assert np.array_equal(back, nkept[:, None] * d["x"])


@pytest.mark.parametrize("dtype,k", [(I.BF16, 2), (I.F32, 1)])
def test_dispatch_from_the_slot_side_and_from_the_token_side_agree(dtype, k):
    """moe_dispatch (one wave per slot, source looked up in slot_src) and moe_dispatch_tokens (one wave per
    token, destinations from expert_idx / slot) fill the rows in use with the same bit copies of x; neither
    touches a row that is not in use."""
    w = I.small("dispatch2", 1500, 72, 64, 7, k, 430 if k == 2 else 260, dtype, skew="hot0", skew_param=0.5)   # some experts overflow, others underfill
    d = I.make_inputs(w, seed=23)
    d["Wg"] = d["Wg"] * 8.0
    layer, got = G.run_layer(w, d)
    x = G.to_dev(d["x"], w.dtype)
    fill = 7.0
    a = torch.full_like(layer.xd, fill)
    b = torch.full_like(layer.xd, fill)
    B.moe_dispatch(layer.shape, x, layer.slot_src, layer.expert_count, a)
    B.moe_dispatch_tokens(layer.shape, x, layer.expert_idx, layer.slot, b)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    a = G.host(a)
    m = G.row_mask(got["expert_count"], w.capacity)
    assert (got["slot"] < 0).any() and m.any() and not m.all()
    assert np.array_equal(a[m], d["x"][got["slot_src"][m] // w.k])
    assert np.all(a[~m] == fill)


def test_two_runs_are_bit_identical():
    w = I.small("determinism", 2000, 128, 256, 8, 2, 450, I.BF16)
    d = I.make_inputs(w, seed=19)
    _, a = G.run_layer(w, d)
    _, b = G.run_layer(w, d)
    m = G.row_mask(a["expert_count"], w.capacity)
    for n in a:
        if a[n].ndim == 3 and a[n].shape[:2] == m.shape:
            assert np.array_equal(a[n][m], b[n][m]), n
        else:
            assert np.array_equal(a[n], b[n]), n


@pytest.mark.parametrize("T,d,E", [(1, 8, 36), (100, 72, 64), (129, 264, 100), (1000, 1024, 128), (5000, 200, 128),
                                   (25000, 136, 44), (2049, 320, 33), (700, 64, 130), (300, 1032, 256)])
@pytest.mark.parametrize("with_bias", [False, True])
def test_gate_projection_with_many_experts(T, d, E, with_bias):
    """bf16 activations and more than 32 experts: the projection is tiled like a GEMM (expert counts that are a
    multiple of 4 up to 128) or runs per 32/64 tokens (the others).  Ragged token counts, reduction lengths that are
    no multiple of the slab, one and several workgroups, both workgroup sizes; every logit against the oracle, per
    row as well, and rows next to the output untouched."""
    w = I.small("proj", T, d, 8, E, 1, 4, I.BF16, w_std=0.5)
    data = I.make_inputs(w, seed=T + E)
    if not with_bias:
        data["bias"] = None
    else:
        data["bias"] = np.linspace(-1.0, 1.0, E).astype(np.float32)
    ref64, _ = G.oracle_logits(dict(data, bias=data["bias"] if with_bias else np.zeros(E, np.float32)))
    shape = B.make_shape(T, d, 8, E, 1, 4, I.BF16, 0)
    lg = torch.full((T + 2, E), 7.0, device="cuda")
    print(f"[gpu] projection T={T} d={d} E={E} bias={with_bias}", flush=True)
    B.moe_gate_logits(shape, G.to_dev(data["x"], I.BF16), G.to_dev(data["Wg"], I.F32),
                      G.to_dev(data["bias"], I.F32), lg[1:T + 1])
    torch.cuda.synchronize()
    got = G.host(lg)
    assert (got[0] == 7.0).all() and (got[T + 1] == 7.0).all()
    assert G.rel_l2(got[1:T + 1], ref64) <= 1e-5
    G.assert_rows("logits", got[1:T + 1], ref64, 1e-5)


def test_argument_errors_leave_outputs_untouched():
    w = I.small("err", 64, 16, 16, 4, 1, 16)
    s = B.make_shape(w.T, w.d_model, w.d_ff, w.E, w.k, w.capacity, w.dtype, w.act)
    logits = torch.zeros(64, 4, device="cuda")
    x = torch.zeros(64, 16, device="cuda")
    Wg = torch.zeros(16, 4, device="cuda")
    with pytest.raises(B.MoeError, match="NULL"):
        B.moe_gate_logits(s, x, None, None, logits)
    bad = B.make_shape(64, 12, 16, 4, 1, 16, 0, 0)           # d_model not a multiple of 8
    sentinel = torch.full((64, 4), 7.0, device="cuda")
    with pytest.raises(B.MoeError, match="shape"):
        B.moe_gate_logits(bad, x, Wg, None, sentinel)
    torch.cuda.synchronize()
    assert torch.all(sentinel == 7.0)
    ws_small = torch.empty(256, dtype=torch.uint8, device="cuda")
    i32 = lambda *sh: torch.empty(sh, dtype=torch.int32, device="cuda")
    with pytest.raises(B.MoeError, match="workspace"):
        B.moe_gate_route(s, logits, None, torch.empty(64, 4, device="cuda"), i32(64, 1),
                         torch.empty(64, 1, device="cuda"), i32(64, 1), i32(4), i32(4), i32(4, 16),
                         ws_small)
    # the fused backward call: missing dxd / slot / dx, bad jitter range, short workspace
    ws = torch.empty(B.moe_workspace_bytes(s), dtype=torch.uint8, device="cuda")
    dxd = torch.zeros(4, 16, 16, device="cuda")
    dWg, dx = torch.full((16, 4), 7.0, device="cuda"), torch.full((64, 16), 7.0, device="cuda")
    eidx, slot = torch.zeros(64, 1, dtype=torch.int32, device="cuda"), torch.zeros(64, 1, dtype=torch.int32, device="cuda")
    for args, what in (((s, x, Wg, logits, None, eidx, slot, 0.0, 0, dWg, dx, ws), "NULL"),
                       ((s, x, Wg, logits, dxd, eidx, None, 0.0, 0, dWg, dx, ws), "NULL"),
                       ((s, x, Wg, logits, dxd, eidx, slot, 0.0, 0, dWg, None, ws), "NULL"),
                       ((s, x, Wg, logits, dxd, eidx, slot, 1.5, 0, dWg, dx, ws), "shape"),
                       ((s, x, Wg, logits, dxd, eidx, slot, 0.0, 0, dWg, dx, ws_small[:64]), "workspace")):
        with pytest.raises(B.MoeError, match=what):
            B.moe_dispatch_gate_logits_bwd(*args)
    torch.cuda.synchronize()
    assert torch.all(dWg == 7.0) and torch.all(dx == 7.0)


@pytest.mark.parametrize("T,d,E,k,C,dtype,eps", [
    (777, 136, 5, 2, 200, I.F32, 0.0),        # ragged T and d, E not a multiple of 4
    (1000, 72, 7, 1, 130, I.F32, 0.0),
    (1500, 264, 6, 2, 400, I.BF16, 0.0),
    (2049, 320, 40, 1, 300, I.BF16, 0.0),     # two 32-expert blocks
    (640, 128, 8, 2, 96, I.BF16, 0.05),       # with gate jitter
    (4096, 1024, 32, 2, 512, I.BF16, 0.0),    # cfg3's row length
    # many experts and enough tokens for the 128-token workgroups: ragged T, d no multiple of 64,
    # expert counts that leave the last 16-expert step partly or wholly empty
    (24577, 136, 128, 2, 500, I.BF16, 0.0),
    (25000, 200, 100, 1, 300, I.BF16, 0.0),
    (24600, 72, 36, 2, 900, I.BF16, 0.0),
])
def test_dispatch_backward_fused_with_gate_projection_backward(T, d, E, k, C, dtype, eps):
    """dx = (sum of the token's kept rows of dxd) + dlogits Wg^T in one call, on a
    hand-made assignment: a third of the choices dropped, some tokens without any
    kept choice, every kept choice in a distinct row of its expert."""
    rng = np.random.default_rng(T + d)
    expert_idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    slot = np.full((T, k), -1, np.int32)
    fill = np.zeros(E, np.int64)
    for t in range(T):
        if rng.random() < 0.1:
            continue                                   # token dropped by both experts
        for j in range(k):
            e = expert_idx[t, j]
            if rng.random() < 0.75 and fill[e] < C:
                slot[t, j] = fill[e]
                fill[e] += 1
    # rows in shuffled order inside each expert, so that slots are not monotone in t
    for e in range(E):
        perm = rng.permutation(C)
        m = (expert_idx == e) & (slot >= 0)
        slot[m] = perm[slot[m]]
    x = rng.standard_normal((T, d)).astype(np.float32)
    dxd = rng.standard_normal((E, C, d)).astype(np.float32)
    Wg = (rng.standard_normal((d, E)) * 0.5).astype(np.float32)
    dl = (rng.standard_normal((T, E)) * 0.5).astype(np.float32)
    if dtype == I.BF16:
        x, dxd = I.round_to_bf16(x), I.round_to_bf16(dxd)
    shape = B.make_shape(T, d, 4 * d, E, k, C, dtype, I.GELU)
    ws = torch.empty(B.moe_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    dWg = torch.empty((d, E), dtype=torch.float32, device="cuda")
    dx = G.to_dev(rng.standard_normal((T, d)).astype(np.float32), dtype)     # garbage: must be overwritten
    print(f"[gpu] fused dispatch/gate backward T={T} d={d} E={E} k={k} eps={eps}", flush=True)
    B.moe_dispatch_gate_logits_bwd(shape, G.to_dev(x, dtype), G.to_dev(Wg, I.F32), G.to_dev(dl, I.F32),
                                   G.to_dev(dxd, dtype), G.to_dev(expert_idx, None), G.to_dev(slot, None),
                                   eps, 11, dWg, dx, ws)
    torch.cuda.synchronize()
    noise = O.jitter_noise(T, d, eps, 11) if eps else 1.0
    dWg_ref, dx_gate = O.gate_logits_bwd(x * noise, Wg, dl)
    dx_ref = O.combine_fwd(dxd, expert_idx, slot) + dx_gate * noise
    assert G.rel_l2(G.host(dWg), dWg_ref) <= 1e-5
    assert G.rel_l2(G.host(dx), dx_ref) <= G.TOL[dtype]
    G.assert_rows("dx", G.host(dx), dx_ref, G.TOL[dtype])
    none_kept = (slot < 0).all(axis=1)
    assert none_kept.any()
    assert G.rel_l2(G.host(dx)[none_kept], (dx_gate * noise)[none_kept]) <= G.TOL[dtype]


def test_gate_projection_backward_accumulates_with_many_experts():
    """dx += dlogits Wg^T (no gather) on the 128-token workgroups: ragged T, 64 experts, a preset dx."""
    T, d, E = 24700, 104, 64
    rng = np.random.default_rng(9)
    x = I.round_to_bf16(rng.standard_normal((T, d)).astype(np.float32))
    dx0 = I.round_to_bf16(rng.standard_normal((T, d)).astype(np.float32))
    Wg = (rng.standard_normal((d, E)) * 0.5).astype(np.float32)
    dl = (rng.standard_normal((T, E)) * 0.5).astype(np.float32)
    shape = B.make_shape(T, d, 8, E, 1, 4, I.BF16, I.GELU)
    ws = torch.empty(B.moe_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    dWg = torch.empty((d, E), dtype=torch.float32, device="cuda")
    dx = torch.full((T + 2, d), 3.0, dtype=torch.bfloat16, device="cuda")
    dx[1:T + 1] = G.to_dev(dx0, I.BF16)
    print("[gpu] gate projection backward, accumulate form, 64 experts", flush=True)
    B.moe_gate_logits_bwd(shape, G.to_dev(x, I.BF16), G.to_dev(Wg, I.F32), G.to_dev(dl, I.F32), dWg, dx[1:T + 1], ws)
    torch.cuda.synchronize()
    dWg_ref, dx_ref = O.gate_logits_bwd(x, Wg, dl)
    got = G.host(dx)
    assert (got[0] == 3.0).all() and (got[T + 1] == 3.0).all()
    assert G.rel_l2(G.host(dWg), dWg_ref) <= 1e-5
    assert G.rel_l2(got[1:T + 1], dx0 + dx_ref) <= G.TOL[I.BF16]
    G.assert_rows("dx", got[1:T + 1], dx0 + dx_ref, G.TOL[I.BF16])


def test_mfma_rate_aid_counts_what_it_claims():
    """The measurement aid's work formula (4 waves x iters x 8 MFMAs of 32x32x16 per workgroup) holds: with
    operands 0.5 and 1.0 every accumulator element gains 16 * 0.5 per MFMA, and a lane sums 8 tiles x 16 elements."""
    out = torch.zeros(3 * 256, dtype=torch.float32, device="cuda")
    B.moe_microbench_mfma_bf16(3, 10, 0, out)
    torch.cuda.synchronize()
    assert torch.all(out == 8 * 16 * 8.0 * 10)
    with pytest.raises(B.MoeError):
        B.moe_microbench_mfma_bf16(0, 10, 0, out)


@pytest.mark.parametrize("case", ["ties16", "all_equal", "wide_range", "one_expert"])
def test_long_segments_rank_through_key_buckets(case):
    """Segments of thousands of candidates (skewed routing) take the bucketed ranking path: same slots as the
    oracle's pairwise definition, with massive key ties, identical keys, keys spanning many magnitudes and both
    signs, and every token on one expert."""
    rng = np.random.default_rng(17)
    T, E, k = 12288, 3, 2
    logits = rng.standard_normal((T, E)).astype(np.float32)
    keys = rng.random(T).astype(np.float32)
    if case == "ties16":
        keys = np.floor(keys * 16).astype(np.float32) / 16
    elif case == "all_equal":
        keys[:] = 0.25
    elif case == "wide_range":
        keys = (np.sign(rng.standard_normal(T)) * np.exp(rng.uniform(-60, 60, T))).astype(np.float32)
        keys[::7] = 0.0
    elif case == "one_expert":
        k = 1
        logits[:, 1] += 50.0
    C = 3000
    shape = B.make_shape(T, 64, 128, E, k, C, I.F32, I.RELU)
    ws = torch.empty(B.moe_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
    i32 = lambda *s: torch.empty(s, dtype=torch.int32, device="cuda")
    probs = torch.empty((T, E), dtype=torch.float32, device="cuda")
    gate_w = torch.empty((T, k), dtype=torch.float32, device="cuda")
    eidx, slot, cnt, dem, src = i32(T, k), i32(T, k), i32(E), i32(E), i32(E, C)
    print(f"[gpu] long segments, case {case}", flush=True)
    B.moe_gate_route(shape, G.to_dev(logits, I.F32), G.to_dev(keys, I.F32), probs, eidx, gate_w, slot, cnt, dem, src, ws)
    torch.cuda.synchronize()
    ref_idx = O.top_k(logits, k)
    ref = dict(zip(("slot", "expert_count", "expert_demand", "slot_src"), O.route(ref_idx, keys, E, C)))
    assert np.array_equal(G.host(eidx), ref_idx)
    for name, got in (("slot", slot), ("expert_count", cnt), ("expert_demand", dem), ("slot_src", src)):
        assert np.array_equal(G.host(got), ref[name]), name
    assert ref["expert_demand"].max() > 4 * 256          # the bucketed path was taken
    assert (ref["slot"] < 0).any()                       # and capacity dropped some candidates


def test_step_recorded_as_hip_graph_replays_bit_equal():
    """A step captured into a HIP graph gives, on every replay, exactly what the eager step gives on the same
    inputs - with the inputs refilled in place and eager work of another layer between the replays."""
    from paper_2109_10465_amd.layer import MoELayer
    w = I.small("graph", 1500, 128, 264, 6, 2, 420, I.BF16, I.GELU, skew="hot0", skew_param=0.4)
    outs = ("y", "dx", "dWg", "dW1", "dW2", "slot", "expert_count", "slot_src", "dlogits")
    mk = lambda: MoELayer(w.T, w.d_model, w.d_ff, w.E, w.k, w.capacity, w.dtype, w.act)
    Lg, Le = mk(), mk()
    adt = torch.bfloat16
    d0 = I.make_inputs(w, seed=0)
    t = {n: G.to_dev(d0[n], w.dtype if n in ("x", "dy", "W1", "W2") else I.F32) for n in ("x", "dy", "W1", "W2", "Wg", "bias", "rts_keys")}
    print("[gpu] capturing a step", flush=True)
    graph = Lg.capture_step(t["x"], t["Wg"], t["bias"], t["W1"], t["W2"], t["rts_keys"], t["dy"])
    for seed in (0, 1, 2, 3):
        d = I.make_inputs(w, seed=seed)
        for n in ("x", "dy", "rts_keys"):                       # refilled in place: the graph holds the addresses
            t[n].copy_(G.to_dev(d[n], w.dtype if n != "rts_keys" else I.F32))
        for name in outs:                                       # stale results must not survive
            getattr(Lg, name).fill_(-7)
        print(f"[gpu] replay with inputs of seed {seed}", flush=True)
        graph.replay()
        Le.step(t["x"], t["Wg"], t["bias"], t["W1"], t["W2"], t["rts_keys"], t["dy"])
        torch.cuda.synchronize()
        kept = G.row_mask(G.host(Le.expert_count), w.capacity)
        for name in outs:
            a, b = getattr(Lg, name), getattr(Le, name)
            assert torch.equal(a, b), (seed, name)
        assert adt == Lg.y.dtype and kept.any()


@pytest.mark.parametrize("E,k", [(12, 2), (130, 2), (5, 1)])
def test_non_finite_logits_and_keys_keep_every_index_in_range(E, k):
    """The ABI promises no fault for non-finite logits or keys (the values are then undefined).
    A row of NaN logits never wins a comparison; the selection treats NaN as -inf, so the
    chosen ids stay valid and distinct and everything indexed with them stays in bounds."""
    T, C, dm = 1000, 150, 64
    rng = np.random.default_rng(3)
    lg = (rng.standard_normal((T, E)) * 2).astype(np.float32)
    keys = rng.random(T, dtype=np.float32)
    clean = lg.copy()
    lg[3] = np.nan
    lg[500] = np.nan
    lg[10, 1] = np.nan
    lg[11, :2] = np.inf
    lg[12] = -np.inf
    keys[[5, 6, 700]] = np.nan
    keys[8] = np.inf
    keys[9] = -np.inf
    s = B.make_shape(T, dm, dm, E, k, C, I.F32, I.RELU)
    dev = lambda a: torch.from_numpy(a).cuda()
    i32, f32 = torch.int32, torch.float32
    out = dict(probs=torch.empty((T, E), dtype=f32, device="cuda"), expert_idx=torch.full((T, k), -9, dtype=i32, device="cuda"),
               gate_w=torch.empty((T, k), dtype=f32, device="cuda"), slot=torch.full((T, k), -9, dtype=i32, device="cuda"),
               expert_count=torch.empty((E,), dtype=i32, device="cuda"), expert_demand=torch.empty((E,), dtype=i32, device="cuda"),
               slot_src=torch.full((E, C), 0x7ffffff0, dtype=i32, device="cuda"))     # a wild value wherever nothing is written
    ws = torch.empty(B.moe_workspace_bytes(s), dtype=torch.uint8, device="cuda")
    print(f"[gpu] non-finite routing inputs: T={T} E={E} k={k} C={C}", flush=True)
    B.moe_gate_route(s, dev(lg), dev(keys), out["probs"], out["expert_idx"], out["gate_w"], out["slot"],
                     out["expert_count"], out["expert_demand"], out["slot_src"], ws)
    torch.cuda.synchronize()
    e = out["expert_idx"].cpu().numpy()
    sl = out["slot"].cpu().numpy()
    src = out["slot_src"].cpu().numpy()
    assert ((e >= 0) & (e < E)).all()
    if k == 2:
        assert (e[:, 0] != e[:, 1]).all()
    # NaN keys can give two candidates of an expert the same rank: a slot below expert_count may then stay
    # unwritten (dispatch skips whatever is not a candidate id); everything that IS written is in range
    assert ((sl >= -1) & (sl < C)).all() and (((src >= -1) & (src < T * k)) | (src == 0x7ffffff0)).all()
    cnt = out["expert_count"].cpu().numpy()
    assert ((cnt >= 0) & (cnt <= C)).all() and int(out["expert_demand"].sum()) == T * k
    # rows without a NaN choose what the definition says (NaN counts as -inf, so row 10 is defined too)
    ref = O.top_k(np.where(np.isnan(lg), -np.inf, lg)[[0, 1, 2, 10, 999]], k)
    assert np.array_equal(e[[0, 1, 2, 10, 999]], ref)
    assert np.array_equal(e[[3, 500]], np.tile(np.arange(k), (2, 1)))       # all-NaN rows: the smallest ids
    # the consumers of these indices run on them without leaving their buffers
    x = torch.from_numpy(rng.standard_normal((T, dm)).astype(np.float32)).cuda()
    xd = torch.zeros((E, C, dm), dtype=f32, device="cuda")
    y = torch.empty((T, dm), dtype=f32, device="cuda")
    dl = torch.empty((T, E), dtype=f32, device="cuda")
    B.moe_dispatch(s, x, out["slot_src"], out["expert_count"], xd)
    B.moe_combine_fwd(s, xd, out["expert_idx"], out["slot"], out["gate_w"], y)
    B.moe_gate_bwd(s, out["gate_w"], out["probs"], out["expert_idx"], out["slot"], dl)
    torch.cuda.synchronize()
    assert np.isfinite(clean).all()
