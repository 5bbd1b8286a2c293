"""GPU parity of the seeded training noise — gate jitter (Sec. 5.1) and expert
dropout (Sec. 5.4) — through the C ABI against the CPU oracle.  Both sides
implement the same counter-based generator, so every draw is reproduced."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2109_10465_amd import binding as B
from paper_2109_10465_amd import inputs as I

import gpu_util as G

pytestmark = pytest.mark.gpu

CASES = [
    (I.small("noise_f32_top1", 1000, 72, 136, 7, 1, 180, I.F32, I.GELU, skew="hot0", skew_param=0.4), 0.01, 0.4),
    (I.small("noise_f32_top2", 777, 136, 264, 5, 2, 250, I.F32, I.RELU, skew="hot0", skew_param=0.5), 0.05, 0.1),
    (I.small("noise_bf16_top2", 1500, 264, 520, 6, 2, 420, I.BF16, I.GELU, skew="zipf", skew_param=1.1), 0.01, 0.4),
    (I.small("noise_bf16_manyE", 2048, 64, 72, 100, 2, 60, I.BF16, I.GELU), 0.02, 0.25),
    (I.small("jitter_only", 600, 40, 72, 5, 2, 300, I.F32, I.GELU), 0.01, 0.0),
    (I.small("dropout_only", 600, 40, 72, 5, 2, 300, I.BF16, I.GELU), 0.0, 0.4),
]
SEED = (0x1234 << 32) | 0x9abcdef1      # both key words in use


@pytest.mark.parametrize("w,eps,p", CASES, ids=lambda v: v.name if hasattr(v, "name") else str(v))
def test_layer_with_jitter_and_dropout(w, eps, p):
    d = I.make_inputs(w, seed=19)
    d["Wg"] = d["Wg"] * 8.0
    ref64, lg32 = G.oracle_logits(d, eps, SEED)
    ref = O.moe_layer(d["x"], d["Wg"], d["bias"], d["W1"], d["W2"], d["rts_keys"], d["dy"], w.k, w.capacity, w.act,
                      logits=lg32, jitter_eps=eps, drop_p=p, seed=SEED)
    _, got = G.run_layer(w, d, logits=lg32, jitter_eps=eps, drop_p=p, seed=SEED)
    sc = O.dropout_scale(w.E, w.capacity, w.d_ff, p, SEED) if p > 0 else None
    errs = G.compare_full(w, d, got, ref, scale=sc)
    # the GPU's own jittered projection
    _, chained = G.run_layer(w, d, jitter_eps=eps, drop_p=p, seed=SEED)
    assert G.rel_l2(chained["logits"], ref64) <= 1e-5
    G.check_chained_routing(w, d, chained, lg32, ref)
    if p > 0:       # the mask itself: dropped elements are exact zeros, kept ones are not (bar gelu(0))
        m = G.row_mask(ref["expert_count"], w.capacity)
        assert not got["h"][m][sc[m] == 0].any() and not got["dact"][m][sc[m] == 0].any()
        live = O.act_grad(ref["Z"], w.act)[m] != 0        # relu'(z) is zero on its own for z <= 0
        assert np.array_equal((got["dact"][m] != 0)[live], (sc[m] > 0)[live])
    if eps > 0:
        plain64, _ = G.oracle_logits(d)
        assert G.rel_l2(chained["logits"], plain64) > 1e-4       # the jitter is really there
    print(w.name, {k: f"{v:.1e}" for k, v in errs.items() if k in ("y", "dx", "dWg", "dW1")})


def test_zero_noise_entry_points_equal_the_plain_ones_bit_for_bit():
    w = I.small("noise_off", 512, 64, 136, 6, 2, 200, I.BF16, I.GELU)
    d = I.make_inputs(w, seed=3)
    _, a = G.run_layer(w, d)
    _, b = G.run_layer(w, d, jitter_eps=0.0, drop_p=0.0, seed=SEED)
    for n in ("logits", "y", "dx", "dWg", "dW1", "dW2"):
        assert np.array_equal(a[n], b[n]), n


def test_noise_argument_errors():
    shape = B.make_shape(256, 16, 16, 4, 1, 64, B.F32, 0)
    t = lambda shp, dt=torch.float32: torch.zeros(shp, dtype=dt, device="cuda")
    x, Wg, lg = t((256, 16)), t((16, 4)), t((256, 4))
    for bad in (-0.1, 1.0, float("nan")):
        with pytest.raises(B.MoeError):
            B.moe_gate_logits_jitter(shape, x, Wg, None, bad, 1, lg)
    xd, W1, W2 = t((4, 64, 16)), t((4, 16, 16)), t((4, 16, 16))
    cnt = torch.full((4,), 64, dtype=torch.int32, device="cuda")
    h, a, yd = t((4, 64, 16)), t((4, 64, 16)), t((4, 64, 16))
    for bad in (-0.5, 1.0, float("nan")):
        with pytest.raises(B.MoeError):
            B.moe_expert_ffn_fwd_dropout(shape, xd, cnt, W1, W2, bad, 1, h, a, yd)
    with pytest.raises(B.MoeError):      # dropout without the saved derivative
        B.moe_expert_ffn_fwd_dropout(shape, xd, cnt, W1, W2, 0.4, 1, h, None, yd)
    B.moe_expert_ffn_fwd_dropout(shape, xd, cnt, W1, W2, 0.4, 1, h, a, yd)


def test_full_size_cfg3_jittered_projection_and_dropout_forward():
    """cfg3 at full size: the jittered gate projection against the oracle in full,
    and the dropout forward GEMM on sampled columns of two experts over all their rows."""
    w = I.WORKLOADS["cfg3"]
    d = I.make_inputs(w, seed=0)
    eps, p = 0.01, 0.4
    shape = B.make_shape(w.T, w.d_model, w.d_ff, w.E, w.k, w.capacity, w.dtype, w.act)
    ref64, _ = G.oracle_logits(d, eps, SEED)
    x = G.to_dev(d["x"], w.dtype)
    lg = torch.empty((w.T, w.E), device="cuda")
    print("[gpu] cfg3 jittered projection", flush=True)
    B.moe_gate_logits_jitter(shape, x, G.to_dev(d["Wg"], I.F32), G.to_dev(d["bias"], I.F32), eps, SEED, lg)
    torch.cuda.synchronize()
    assert G.rel_l2(G.host(lg), ref64) <= 1e-5
    # dropout forward on generator-made expert inputs: the first rows of x serve as every expert's xd
    rng = np.random.default_rng(3)
    cnt = rng.integers(w.capacity // 2, w.capacity + 1, size=w.E).astype(np.int32)
    xd_host = d["x"][: w.capacity]
    xd = G.to_dev(np.broadcast_to(xd_host, (w.E, w.capacity, w.d_model)).copy(), w.dtype)
    W1, W2 = G.to_dev(d["W1"], w.dtype), G.to_dev(d["W2"], w.dtype)
    h = torch.empty((w.E, w.capacity, w.d_ff), dtype=torch.bfloat16, device="cuda")
    a, yd = torch.empty_like(h), torch.empty((w.E, w.capacity, w.d_model), dtype=torch.bfloat16, device="cuda")
    print("[gpu] cfg3 dropout forward", flush=True)
    B.moe_expert_ffn_fwd_dropout(shape, xd, torch.from_numpy(cnt).cuda(), W1, W2, p, SEED, h, a, yd)
    torch.cuda.synchronize()
    thr = int(np.floor(p * 2.0 ** 32))
    for e in (0, w.E - 1):
        n = int(cnt[e])
        cols = np.sort(rng.choice(w.d_ff, size=32, replace=False))
        Z = np.asarray(xd_host[:n], np.float64) @ np.asarray(d["W1"][e][:, cols], np.float64)
        # words of elements (e, s, c): index (e*C + s)*f + c, taken from the oracle's generator block by block
        idx = ((e * w.capacity + np.arange(n))[:, None] * w.d_ff + cols[None, :]).astype(np.uint64)
        blk = idx >> np.uint64(2)
        words = np.stack(O.philox4x32(blk & np.uint64(0xFFFFFFFF), blk >> np.uint64(32), O.STREAM_DROPOUT, 0,
                                      SEED & 0xFFFFFFFF, SEED >> 32), axis=-1)
        word = np.take_along_axis(words, (idx & np.uint64(3)).astype(np.int64)[..., None], axis=-1)[..., 0]
        sc = (word >= thr) / (1.0 - p)
        assert G.rel_l2(G.host(h[e, :n])[:, cols], O.act(Z, w.act) * sc) <= G.TOL[w.dtype]
        assert G.rel_l2(G.host(a[e, :n])[:, cols], O.act_grad(Z, w.act) * sc) <= G.TOL[w.dtype]
        assert np.array_equal(G.host(a[e, :n])[:, cols] != 0, sc > 0)
