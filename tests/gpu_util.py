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


def assert_rows(name, got, want, tol):
    """Per-row bound that goes with the whole-tensor rel-L2 bound `tol`: a tensor-wide norm lets a few entirely
    wrong rows of a large tensor through (one row of 16384 weighs 0.8 % of the norm).  Every row (last axis) must be
    within row_tol of the oracle's row, relative to the row's norm or, for rows that are small against the typical
    one (sums that cancel), to the median row norm; and no element may be off by more than 2*row_tol of the largest
    magnitude in the tensor.  row_tol = 2*tol for bf16 (4e-2); for fp32 it is 1e-3: single rows of fp32 results
    that come from cancelling sums (a gate gradient scaled by a small dot product) legitimately sit 10-100x above
    the tensor-wide 1e-5, while a wrong row is off by order one."""
    g = np.asarray(got, np.float64)
    w_ = np.asarray(want, np.float64)
    assert g.shape == w_.shape, (name, g.shape, w_.shape)
    if w_.size == 0:
        return
    g = g.reshape(-1, g.shape[-1]) if g.ndim > 1 else g.reshape(-1, 1)
    w_ = w_.reshape(g.shape)
    rn = np.linalg.norm(w_, axis=1)
    dn = np.linalg.norm(g - w_, axis=1)
    nz = rn[rn > 0]
    floor = np.median(nz) if nz.size else 0.0
    row_tol = max(2.0 * tol, 1e-3)
    bad = dn > row_tol * np.maximum(rn, floor) + 1e-30
    assert not bad.any(), (name, "rows", np.nonzero(bad)[0][:8].tolist(), float((dn / np.maximum(rn, floor + 1e-300)).max()))
    amax = float(np.abs(w_).max())
    assert float(np.abs(g - w_).max()) <= 2.0 * row_tol * amax + 1e-30, (name, "max abs", float(np.abs(g - w_).max()), amax)


def run_layer(w, d, use_keys=True, logits=None, aux_coef=0.0, groups=1, jitter_eps=0.0, drop_p=0.0, seed=0):
    """One forward+backward of workload w on the GPU; returns (layer, dict of
    host arrays) with the same names the oracle uses.  logits (fp32 numpy, made
    by the oracle) replaces the GPU's gate projection as the router's input."""
    layer = MoELayer(w.T, w.d_model, w.d_ff, w.E, w.k, w.capacity, w.dtype, w.act, aux_coef=aux_coef, groups=groups,
                     jitter_eps=jitter_eps, drop_p=drop_p)
    x, dy = to_dev(d["x"], w.dtype), to_dev(d["dy"], w.dtype)
    W1, W2 = to_dev(d["W1"], w.dtype), to_dev(d["W2"], w.dtype)
    Wg = to_dev(d["Wg"], I.F32)
    bias = to_dev(d["bias"], I.F32)
    keys = to_dev(d["rts_keys"], I.F32) if use_keys else None
    print(f"[gpu] {w.name}: T={w.T} d={w.d_model} f={w.d_ff} E={w.E} k={w.k} C={w.capacity} "
          f"dtype={w.dtype} keys={use_keys} logits={'gpu' if logits is None else 'given'}", flush=True)
    layer.step(x, Wg, bias, W1, W2, keys, dy, None if logits is None else to_dev(logits, I.F32), seed)
    torch.cuda.synchronize()
    names = ["logits", "probs", "expert_idx", "gate_w", "slot", "expert_count", "expert_demand",
             "slot_src", "xd", "h", "dact", "yd", "y", "dyd", "dgate_w", "dxd", "dW1", "dW2",
             "dlogits", "dWg", "dx"]
    if aux_coef != 0.0:
        names += ["first_frac", "mean_prob", "aux_loss"]
    out = {n: host(getattr(layer, n)) for n in names}
    return layer, out


def oracle_logits(d, jitter_eps=0.0, seed=0):
    """The oracle's gate logits in fp64 and rounded to fp32, the precision in
    which both sides take the top-k decision."""
    xg = np.asarray(d["x"], np.float64)
    if jitter_eps != 0.0:
        xg = xg * O.jitter_noise(xg.shape[0], xg.shape[1], jitter_eps, seed)
    ref64 = O.gate_logits(xg, d["Wg"], d["bias"])
    return ref64, ref64.astype(np.float32)


def check_chained_routing(w, d, got, lg32, ref_route, use_keys=True):
    """The chained path (GPU projection -> GPU router) against the oracle's
    routing.  fp32 matmuls differ in their last bits between CPU and GPU, which
    can flip the top-k choice of a token whose relevant logits are closer than
    that error; such tokens have more than one correct answer.  Every other
    token must match exactly; for the near-tied ones the GPU's choice must be
    within the error of the oracle's, and the slots must then be the ones the
    capacity rule gives for that choice.  Returns the number of near-tied tokens."""
    assert rel_l2(got["logits"], lg32) <= 1e-5
    err = float(np.max(np.abs(got["logits"].astype(np.float64) - lg32))) if lg32.size else 0.0
    thr = 4.0 * err + 1e-30
    srt = -np.sort(-lg32.astype(np.float64), axis=1)
    ngap = min(w.k, w.E - 1)                       # gaps that decide membership and order
    amb = np.zeros(w.T, bool)
    for j in range(ngap):
        amb |= (srt[:, j] - srt[:, j + 1]) < thr
    ref_e = ref_route["expert_idx"]
    assert np.array_equal(got["expert_idx"][~amb], ref_e[~amb])
    if not amb.any():
        for n in INT_NAMES:
            assert np.array_equal(got[n], ref_route[n]), n
        return 0
    rows = np.nonzero(amb)[0]
    ge = got["expert_idx"][rows]
    assert np.all((ge >= 0) & (ge < w.E))
    if w.k == 2:
        assert np.all(ge[:, 0] != ge[:, 1])
    for j in range(w.k):
        assert np.all(lg32[rows, ge[:, j]] >= lg32[rows, ref_e[rows, j]] - thr)
    keys = d["rts_keys"] if use_keys else None
    slot, count, demand, slot_src = O.route(got["expert_idx"], keys, w.E, w.capacity)
    for n, v in (("slot", slot), ("expert_count", count), ("expert_demand", demand), ("slot_src", slot_src)):
        assert np.array_equal(got[n], v), n
    return int(amb.sum())


def row_mask(count, C):
    """[E,C] mask of the rows in use."""
    return np.arange(C)[None, :] < np.asarray(count)[:, None]


def compare_full(w, d, got, ref, aux=False, scale=None):
    """Element-by-element comparison of every output of one GPU run with the
    oracle's: integers bit-exact, floats by rel-L2.  Returns the errors."""
    tol = TOL[w.dtype]
    for n in INT_NAMES:
        assert np.array_equal(got[n], ref[n]), n
    errs = {}
    for n in ["probs", "gate_w"]:
        errs[n] = rel_l2(got[n], ref[n])
        assert errs[n] <= 1e-5, (n, errs[n])
    m = row_mask(ref["expert_count"], w.capacity)
    dact = O.act_grad(ref["Z"], w.act)          # the derivative the forward saves
    if scale is not None:                       # expert dropout folds its factor into it
        dact = dact * scale
    pairs = [("xd", ref["Xd"]), ("h", ref["H"]), ("dact", dact), ("yd", ref["Yd"]), ("dyd", ref["dYd"]),
             ("dxd", ref["dXd"])]
    for g, r in pairs:
        errs[g] = rel_l2(got[g][m], r[m])
        assert errs[g] <= tol, (g, errs[g])
        assert_rows(g, got[g][m], r[m], tol)
    assert np.array_equal(got["xd"][m], d["x"][ref["slot_src"][m] // w.k])     # bit copies
    for n in ["y", "dgate_w", "dW1", "dW2", "dlogits", "dWg", "dx"]:
        errs[n] = rel_l2(got[n], ref[n])
        assert errs[n] <= tol, (n, errs[n])
        assert_rows(n, got[n], ref[n], tol)
    dropped = np.all(ref["slot"] < 0, axis=1)
    assert not got["y"][dropped].any()
    if not aux:     # the balancing loss reaches dropped tokens too
        assert not got["dlogits"][dropped].any() and not got["dx"][dropped].any()
    return errs


def check_full(w, d, got, use_keys=True):
    """Element-by-element parity of every output against the oracle.

    The oracle computes the gate logits in fp64 and rounds them to fp32; its whole
    layer is evaluated from those.  (1) The GPU's projection is compared with
    them (rel-L2 <= 1e-5).  (2) The GPU layer is run with the oracle's fp32 logits
    as the router's input, so both sides take every decision on identical values:
    routing bit-exact, floats by rel-L2.  (3) `got`, the chained run with the
    GPU's own projection, must route identically except on near-tied tokens (see
    check_chained_routing) and, when there are none, match every float as well."""
    keys = d["rts_keys"] if use_keys else None
    _, lg32 = oracle_logits(d)
    ref = O.moe_layer(d["x"], d["Wg"], d["bias"], d["W1"], d["W2"], keys, d["dy"], w.k, w.capacity,
                      w.act, logits=lg32)
    _, staged = run_layer(w, d, use_keys, logits=lg32)
    assert np.array_equal(staged["logits"], lg32)
    errs = compare_full(w, d, staged, ref)
    if check_chained_routing(w, d, got, lg32, ref, use_keys) == 0:
        compare_full(w, d, got, ref)
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
    """Parity of a full-size run on sampled outputs.  `got` is a run routed on
    the oracle's fp32 logits and holds the small tensors in full (logits, probs,
    routing, gate_w, y, dgate_w, dlogits, dWg, dx); per-expert tensors come
    through fetch_expert(name, e) -> host array of expert e.  Returns the worst
    rel-L2 per quantity and the oracle's routing."""
    tol = TOL[w.dtype]
    rng = np.random.default_rng(seed)
    _, lg = oracle_logits(d)
    assert np.array_equal(got["logits"], lg)      # the run was routed on the oracle's fp32 logits
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
        assert_rows(name, a, b, tol)

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
    # dWg sums over every token, which the oracle cannot afford at this size.  A
    # property that holds at any size ties it to dlogits, whose sampled rows are
    # checked above: dWg = x^T dlogits, evaluated here in fp64 on the run's own
    # dlogits.  (The kernel itself is compared with the oracle at full size on
    # generator-made dlogits in its own test.)
    dWg_lin = np.asarray(d["x"], np.float64).T @ np.asarray(got["dlogits"], np.float64)
    upd("dWg", got["dWg"], dWg_lin)
    for n, v in errs.items():
        assert v <= tol, (n, v)
    return errs, route
