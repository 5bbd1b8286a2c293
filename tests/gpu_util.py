"""Helpers shared by the GPU parity tests: upload seeded inputs, run the HIP
layer through the C ABI, download results, compare against the CPU oracle."""
import numpy as np
import torch

from oracle import moe_oracle as O
from paper_2109_10465_amd import binding as B
from paper_2109_10465_amd import inputs as I
from paper_2109_10465_amd.layer import MoELayer

TOL = {I.F32: 1e-5, I.BF16: 2e-2}     # rel-L2 bounds on outputs and gradients
INT_NAMES = ["expert_idx", "slot", "expert_count", "expert_demand", "slot_src"]


def to_dev(a, dtype):
    """fp32 numpy array -> device tensor in the activation dtype (values are
    already bf16-representable for bf16 workloads, so this is exact)."""
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(torch.bfloat16) if dtype == I.BF16 else t


def host(t):
    return t.detach().float().cpu().numpy() if t.dtype.is_floating_point else t.detach().cpu().numpy()


def rel_l2(got, want):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    den = np.linalg.norm(want)
    num = np.linalg.norm(got - want)
    return num / den if den > 0 else num


def run_layer(w, d, use_keys=True):
    """One forward+backward of workload w on the GPU; returns (layer, dict of
    host arrays) with the same names the oracle uses."""
    layer = MoELayer(w.T, w.d_model, w.d_ff, w.E, w.k, w.capacity, w.dtype, w.act)
    x, dy = to_dev(d["x"], w.dtype), to_dev(d["dy"], w.dtype)
    W1, W2 = to_dev(d["W1"], w.dtype), to_dev(d["W2"], w.dtype)
    Wg = to_dev(d["Wg"], I.F32)
    bias = to_dev(d["bias"], I.F32)
    keys = to_dev(d["rts_keys"], I.F32) if use_keys else None
    print(f"[gpu] {w.name}: T={w.T} d={w.d_model} f={w.d_ff} E={w.E} k={w.k} C={w.capacity} "
          f"dtype={w.dtype} keys={use_keys}", flush=True)
    layer.step(x, Wg, bias, W1, W2, keys, dy)
    torch.cuda.synchronize()
    names = ["logits", "probs", "expert_idx", "gate_w", "slot", "expert_count", "expert_demand",
             "slot_src", "xd", "h", "dact", "yd", "y", "dyd", "dgate_w", "dxd", "dW1", "dW2",
             "dlogits", "dWg", "dx"]
    out = {n: host(getattr(layer, n)) for n in names}
    return layer, out


def row_mask(count, C):
    """[E,C] mask of the rows in use."""
    return np.arange(C)[None, :] < np.asarray(count)[:, None]


def check_full(w, d, got, use_keys=True):
    """Element-by-element parity of every output against the oracle.  Routing
    is checked bit-exactly given the GPU's own fp32 logits; floats by rel-L2."""
    tol = TOL[w.dtype]
    keys = d["rts_keys"] if use_keys else None
    ref_logits = O.gate_logits(d["x"], d["Wg"], d["bias"])
    assert rel_l2(got["logits"], ref_logits) <= 1e-5
    ref = O.moe_layer(d["x"], d["Wg"], d["bias"], d["W1"], d["W2"], keys, d["dy"], w.k, w.capacity,
                      w.act, logits=got["logits"])
    for n in INT_NAMES:
        assert np.array_equal(got[n], ref[n]), n
    errs = {}
    for n in ["probs", "gate_w"]:
        errs[n] = rel_l2(got[n], ref[n])
        assert errs[n] <= 1e-5, (n, errs[n])
    m = row_mask(ref["expert_count"], w.capacity)
    ref["dact"] = O.act_grad(ref["Z"], w.act)          # the derivative the forward saves
    pairs = [("xd", "Xd"), ("h", "H"), ("dact", "dact"), ("yd", "Yd"), ("dyd", "dYd"), ("dxd", "dXd")]
    for g, r in pairs:
        errs[g] = rel_l2(got[g][m], ref[r][m])
        assert errs[g] <= tol, (g, errs[g])
    assert np.array_equal(got["xd"][m], d["x"][ref["slot_src"][m] // w.k])     # bit copies
    for n in ["y", "dgate_w", "dW1", "dW2", "dlogits", "dWg", "dx"]:
        errs[n] = rel_l2(got[n], ref[n])
        assert errs[n] <= tol, (n, errs[n])
    dropped = np.all(ref["slot"] < 0, axis=1)
    assert not got["y"][dropped].any()
    assert not got["dlogits"][dropped].any() and not got["dx"][dropped].any()
    return ref, errs


# ---------------------------------------------------------------------------
# full-size workloads: parity on sampled outputs the oracle computes one by one
# ---------------------------------------------------------------------------
class F64Experts:
    """Per-expert fp64 copies of a weight tensor, converted once and cached."""

    def __init__(self, W):
        self.W, self.cache = W, {}

    def __getitem__(self, e):
        if e not in self.cache:
            self.cache[e] = np.asarray(self.W[e], np.float64)
        return self.cache[e]


def oracle_token(t, d, w, route, p_row, g_row):
    """Everything the layer produces for token t, from the definitions, given the
    routing: y[t], dgate_w[t], dlogits[t], dx[t]."""
    k = w.k
    x_t = np.asarray(d["x"][t:t + 1], np.float64)
    dy_t = np.asarray(d["dy"][t:t + 1], np.float64)
    y = np.zeros_like(x_t)
    dx = np.zeros_like(x_t)
    dg = np.zeros((1, k))
    one = np.ones(1, np.int32)
    for j in range(k):
        if route["slot"][t, j] < 0:
            continue
        e = int(route["expert_idx"][t, j])
        W1e, W2e = d["W1"][e][None], d["W2"][e][None]
        Z, H, Yd = O.expert_ffn_fwd(x_t[None], one, W1e, W2e, w.act)
        y += g_row[j] * Yd[0]
        dg[0, j] = float(np.vdot(dy_t, Yd[0]))
        dXd, _, _ = O.expert_ffn_bwd((g_row[j] * dy_t)[None], x_t[None], Z, one, W1e, W2e, w.act)
        dx += dXd[0]
    dl = O.gate_bwd(dg, p_row[None, :], route["expert_idx"][t:t + 1], route["slot"][t:t + 1])
    _, dx_gate = O.gate_logits_bwd(x_t, d["Wg"], dl)
    return y[0], dg[0], dl[0], dx[0] + dx_gate[0]


def oracle_expert_columns(e, cols, d, w, route, gate_w):
    """dW1[e][:, cols] and dW2[e][cols, :] over all rows of expert e, via the
    oracle's FFN on the weight slices (a d_ff = len(cols) expert has exactly
    these weight gradients); also returns the expert's Xd and dYd rows."""
    k = w.k
    n = int(route["expert_count"][e])
    src = route["slot_src"][e, :n]
    tok, j = src // k, src % k
    Xd = np.asarray(d["x"][tok], np.float64)
    dYd = gate_w[tok, j][:, None] * np.asarray(d["dy"][tok], np.float64)
    W1s = np.asarray(d["W1"][e][:, cols], np.float64)[None]
    W2s = np.asarray(d["W2"][e][cols, :], np.float64)[None]
    cnt = np.array([n], np.int32)
    Z, H, _ = O.expert_ffn_fwd(Xd[None], cnt, W1s, W2s, w.act)
    _, dW1, dW2 = O.expert_ffn_bwd(dYd[None], Xd[None], Z, cnt, W1s, W2s, w.act)
    return dW1[0], dW2[0], Xd, dYd, Z[0], H[0]


def check_sampled(w, d, got, n_tokens=192, n_cols=24, n_rows=48, seed=0, fetch_expert=None):
    """Parity of a full-size run on sampled outputs.  `got` holds the small
    tensors in full (logits, probs, routing, gate_w, y, dgate_w, dlogits, dWg,
    dx); per-expert tensors come through fetch_expert(name, e) -> host array of
    expert e.  Returns the worst rel-L2 per quantity."""
    tol = TOL[w.dtype]
    rng = np.random.default_rng(seed)
    ref_logits = O.gate_logits(d["x"], d["Wg"], d["bias"])
    assert rel_l2(got["logits"], ref_logits) <= 1e-5
    lg = got["logits"]
    p = O.softmax(lg)
    eidx = O.top_k(lg, w.k)
    g = O.gate_weights(p, eidx)
    slot, count, demand, slot_src = O.route(eidx, d["rts_keys"], w.E, w.capacity)
    route = dict(expert_idx=eidx, slot=slot, expert_count=count, expert_demand=demand,
                 slot_src=slot_src)
    for n in INT_NAMES:
        assert np.array_equal(got[n], route[n]), n
    assert rel_l2(got["probs"], p) <= 1e-5 and rel_l2(got["gate_w"], g) <= 1e-5
    errs = {}
    d = dict(d, W1=F64Experts(d["W1"]), W2=F64Experts(d["W2"]))

    def upd(name, a, b):
        errs[name] = max(errs.get(name, 0.0), rel_l2(a, b))

    # tokens: a mix of fully kept, partly kept and fully dropped ones
    nk = (slot >= 0).sum(axis=1)
    toks = []
    for c in range(w.k + 1):
        pool = np.nonzero(nk == c)[0]
        if pool.size:
            toks += list(rng.choice(pool, size=min(pool.size, n_tokens // (w.k + 1)), replace=False))
    Y, DG, DL, DX = [], [], [], []
    for t in toks:
        y, dg, dl, dx = oracle_token(int(t), d, w, route, p[t], g[t])
        Y.append(y); DG.append(dg); DL.append(dl); DX.append(dx)
    toks = np.array(toks)
    upd("y", got["y"][toks], np.array(Y))
    upd("dgate_w", got["dgate_w"][toks], np.array(DG))
    upd("dlogits", got["dlogits"][toks], np.array(DL))
    upd("dx", got["dx"][toks], np.array(DX))
    dropped = nk == 0
    assert not got["y"][dropped].any() and not got["dx"][dropped].any()
    assert not got["dlogits"][dropped].any() and not got["dgate_w"][slot < 0].any()
    # experts: most loaded, least loaded non-empty, one more; an empty one if any
    nonempty = np.nonzero(count > 0)[0]
    picks = {int(nonempty[np.argmax(demand[nonempty])]), int(nonempty[np.argmin(count[nonempty])]),
             int(rng.choice(nonempty))}
    for e in sorted(picks):
        cols = np.sort(rng.choice(w.d_ff, size=min(n_cols, w.d_ff), replace=False))
        dW1c, dW2c, Xd, dYd, Zc, Hc = oracle_expert_columns(e, cols, d, w, route, g)
        n = int(count[e])
        upd("dW1", fetch_expert("dW1", e)[:, cols], dW1c)
        upd("dW2", fetch_expert("dW2", e)[cols, :], dW2c)
        xd_e = fetch_expert("xd", e)[:n]
        assert np.array_equal(xd_e, Xd.astype(np.float32))          # bit copies
        upd("dyd", fetch_expert("dyd", e)[:n], dYd)
        upd("dact", fetch_expert("dact", e)[:n][:, cols], O.act_grad(Zc[:n], w.act))
        upd("h", fetch_expert("h", e)[:n][:, cols], Hc[:n])
        rows = np.sort(rng.choice(n, size=min(n_rows, n), replace=False))
        one = np.ones(1, np.int32)
        Ydr, dXdr = [], []
        for r in rows:
            Z, H, Yd = O.expert_ffn_fwd(Xd[r][None, None], one, d["W1"][e][None], d["W2"][e][None], w.act)
            dXd, _, _ = O.expert_ffn_bwd(dYd[r][None, None], Xd[r][None, None], Z, one,
                                         d["W1"][e][None], d["W2"][e][None], w.act)
            Ydr.append(Yd[0, 0]); dXdr.append(dXd[0, 0])
        upd("yd", fetch_expert("yd", e)[rows], np.array(Ydr))
        upd("dxd", fetch_expert("dxd", e)[rows], np.array(dXdr))
    for e in np.nonzero(count == 0)[0][:2]:
        assert not fetch_expert("dW1", int(e)).any() and not fetch_expert("dW2", int(e)).any()
    # dWg = x^T dlogits is linear in dlogits, whose sampled rows are checked above:
    # verify the contraction itself against the GPU's own dlogits in fp64
    dWg_lin, _ = O.gate_logits_bwd(d["x"], d["Wg"], got["dlogits"])
    upd("dWg", got["dWg"], dWg_lin)
    for n, v in errs.items():
        assert v <= tol, (n, v)
    return errs
